// Decoding step against a rank-space KV cache (appendix on decoder models, "Decoding Phase"): one new query per
// sequence attends to the cached rank-space keys and values P_k [t, r_k], P_v [t, r_v] - K and V are never rebuilt.
//
// With q_h = (p_q V_q + b_q)[head h] the score of key j is  q_h . (P_k[j] V_k[:, h] + b_k[h]) =  P_k[j] . w_h + const,
// w_h = V_k[:, h] q_h in R^{r_k} ("absorbed" query; the constant q_h . b_k is the same for every key of the row and
// drops out of the softmax), and the context is  sum_j a_j (P_v[j] V_v[:, h] + b_v[h]) = u_h V_v[:, h] + b_v[h] with
// u_h = sum_j a_j P_v[j] in R^{r_v} (the a_j sum to one).  So the step is two passes over the cache with H vectors on
// each side: S = P_k W^T and U = A P_v, both small matrix products per sequence.  Per sequence and step the kernel
// reads t (r_k + r_v) 2 bytes of cache once for all heads: it is bound by HBM, not by the matrix cores.
//
// Cache layouts (chosen so that a wavefront-wide 16-byte load of 64 consecutive units IS an MFMA operand):
//   K cache, per sequence: the fragment-major layout (fsvd_common.h) of P_k [t_max, r_k].
//   V cache, per sequence: P_v^T in operand order of the U product: for key tile J = key / 32 and rank tile R = rank / 32
//     a 2 KiB block at (J * (r_v / 32) + R) * 2048 (all of a key tile's blocks are contiguous, like its K rows); inside, unit s * 64 + 32 g + (rank % 32) (16 bytes, s = 0..1,
//     g = 0..1) holds the 8 keys 32 J + 16 s + 4 g + {0, 1, 2, 3, 8, 9, 10, 11} of that rank - the contraction-slot
//     order in which the probabilities leave the score accumulators, so they feed the U product without any shuffle.
// Positions that were never written must hold finite values (the caller zero-fills a new cache): masked keys get
// probability exactly 0, and 0 times a non-finite value would not be 0.
#include "fsvd_common.h"
#include "fsvd_kernels.h"

namespace fsvd {

namespace {

constexpr float kLog2eD = 1.4426950408889634f;

// ---------------------------------------------------------------------------------------------------------------
// Cache write: rows P_new [B, n_new, r] (fp16, row-major) -> positions t_start[b] .. of sequence b.  which = 0: K cache
// (one thread per 16-byte unit), which = 1: V cache (one thread per element).  Rows that would fall past t_max are dropped.
// ---------------------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) decode_cache_write_kernel(const _Float16* __restrict__ src, const int32_t* __restrict__ t_start,
                                                                 int B, int t_max, int r, int n_new, int which, _Float16* cache,
                                                                 size_t seq_halves, size_t total) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  if (which == 0) {
    const int groups = r / 8;
    const int rho = 8 * (int)(i % groups);
    const size_t row = i / groups;
    const int n = (int)(row % n_new), b = (int)(row / n_new);
    const int t = t_start[b] + n;
    if (t < 0 || t >= t_max) return;
    const int kch = (r + 63) / 64, off = rho & 63;
    const size_t unit = ((size_t)((t >> 5) * kch + (rho >> 6)) * 4 + ((off >> 3) & 3)) * 64 + (off >> 5) * 32 + (t & 31);
    *(h8*)(cache + b * seq_halves + unit * 8) = *(const h8*)(src + row * r + rho);
  } else {
    const int rho = (int)(i % r);
    const size_t row = i / r;
    const int n = (int)(row % n_new), b = (int)(row / n_new);
    const int t = t_start[b] + n;
    if (t < 0 || t >= t_max) return;
    const int vtl = (r + 31) / 32, kq = t & 31, o = kq & 15;
    const size_t unit = ((size_t)((t >> 5) * vtl + (rho >> 5)) * 2 + (kq >> 4)) * 64 + ((o >> 2) & 1) * 32 + (rho & 31);
    cache[b * seq_halves + unit * 8 + (o & 3) + 4 * (o >> 3)] = src[row * r + rho];
  }
}

// ---------------------------------------------------------------------------------------------------------------
// Absorbed queries: W[b, h, rho] = scale log2(e) * sum_d V_k[rho, h d_h + d] * q[b, h d_h + d], written as the
// fragment-major layout of a [32 (heads, padded), r_k] matrix per sequence (columns of heads >= H are left untouched:
// their scores are never used).  One workgroup per (64 ranks, head), so V_k is read once for the whole batch; the
// product runs on the matrix cores as W^T [ranks, sequences] = V_k[ranks, head columns] q^T: both operands are
// contiguous along d (16-byte loads straight into operand registers).  Wavefront w: rank tile w % 2, sequence tiles
// w / 2, w / 2 + 2, ...
// ---------------------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) decode_absorb_kernel(const _Float16* __restrict__ q, const void* __restrict__ Vk, int w_dt,
                                                            int B, int D, int H, int r_k, float qs, _Float16* W) {
  const int dh = D / H, c = blockIdx.x, h = blockIdx.y;
  const int lane = threadIdx.x & 63, l32 = lane & 31, g = lane >> 5, wave = threadIdx.x >> 6;
  const int rho = 64 * c + 32 * (wave & 1) + l32;
  const int nst = dh / 16;                       // contraction steps (d_h is 64 or 128)
  h8 vf[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    u4 raw = {0u, 0u, 0u, 0u};
    if (s < nst && rho < r_k) raw = *(const u4*)((const uint16_t*)Vk + (size_t)rho * D + h * dh + 16 * s + 8 * g);
    vf[s] = w_dt == DT_BF16 ? raw_to_h8<DT_BF16>(raw) : raw_to_h8<DT_F16>(raw);
  }
  const size_t w_seq = (size_t)((r_k + 63) / 64) * 2048;   // halves per sequence
  for (int bt = wave >> 1; 32 * bt < B; bt += 2) {
    const int b = 32 * bt + l32;
    f16v acc = zero16();
#pragma unroll
    for (int s = 0; s < 8; ++s)
      if (s < nst) {
        h8 qf = {0, 0, 0, 0, 0, 0, 0, 0};
        if (b < B) qf = *(const h8*)(q + (size_t)b * D + h * dh + 16 * s + 8 * g);
        acc = mfma32(vf[s], qf, acc);
      }
    if (b < B) {
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const int off = 32 * (wave & 1) + 8 * jj + 4 * g;          // rank inside the 64-rank chunk, a multiple of 4
        if (64 * c + off < r_k) {
          h4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (_Float16)(acc[4 * jj + e] * qs);
          *(h4*)(W + (size_t)b * w_seq + (size_t)c * 2048 + (((off >> 3) & 3) * 64 + 32 * (off >> 5) + h) * 8 + (off & 7)) = o;
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------------------------
// How the keys of the B sequences are dealt to the G = B * nsplit workgroups of the pass over the cache.  Sequences
// differ in length, so an equal number of parts per sequence leaves the workgroups of short sequences idle while the
// longest one finishes.  Instead every sequence gets parts in proportion to its tiles of 32 keys: with `tpw` a (nearly)
// smallest number of tiles per workgroup for which sum_b parts_b <= G, parts_b = clamp(ceil(tiles_b / tpw), 1, 32),
// sequence b owns the slots first_b .. first_b + parts_b - 1 (first = exclusive prefix sum) and its part s the tiles
// s * ceil(tiles_b / parts_b) ...  Computed by every wavefront for itself from n_keys (lane = sequence, B <= 64; the
// core and the merge kernel must agree, and both evaluate exactly this function); for B > 64 every sequence has
// nsplit parts.  All 64 lanes must call it; lane b < B receives its sequence's values.
// ---------------------------------------------------------------------------------------------------------------
__device__ __forceinline__ int wave_sum(int x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}
__device__ __forceinline__ void decode_parts_of_lane(const int32_t* __restrict__ n_keys, int B, int t_max, int nsplit, int lane,
                                                     int& parts, int& first) {
  if (B > 64) {                           // not balanced: caller indexes by sequence
    parts = nsplit;
    first = 0;
    return;
  }
  const int G = B * nsplit;
  int nt = 0;
  if (lane < B) {
    int n = n_keys[lane];
    n = n < 0 ? 0 : (n > t_max ? t_max : n);
    nt = (n + 31) >> 5;
  }
  const int total = wave_sum(nt);
  // ceil(total / (G - B)) tiles per workgroup always fit (sum_b ceil(tiles_b / tpw) <= total / tpw + B <= G; G >= 4 B here);
  // a few smaller values are tried, the smallest that still fits is kept
  auto parts_at = [&](int t) {
    int q = (nt + t - 1) / t;
    q = q < 1 ? 1 : (q > 32 ? 32 : q);
    return lane < B ? q : 0;
  };
  int tpw = (total + (G - B) - 1) / (G - B);
  tpw = tpw < 1 ? 1 : tpw;
  for (int it = 0; it < 8 && tpw > 1; ++it) {
    if (wave_sum(parts_at(tpw - 1)) > G) break;
    --tpw;
  }
  const int p = parts_at(tpw);
  int incl = p;                           // inclusive prefix sum over the lanes
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int y = __shfl_up(incl, o, 64);
    if (lane >= o) incl += y;
  }
  parts = p;
  first = incl - p;
}

// ---------------------------------------------------------------------------------------------------------------
// The pass over the cache.  One workgroup (8 wavefronts) = one sequence x one part of its keys, all heads at once.
// Per tile of 32 keys:
//   S^T [32 keys, 32 heads] = P_k tile x W^T: the contraction over r_k is split over the wavefronts (64-rank chunks
//   w, w + 8, ..), the partial tiles are exchanged through LDS and every wavefront ends up with the whole tile;
//   mask, streaming softmax per head (head = lane; statistics are per-lane scalars, as in the prefill kernel);
//   U^T [r_v, 32 heads] += (P_v^T tile) x A^T: every wavefront owns the rank tiles w, w + 8, .. of U.
// Operands of the next key tile are requested before the current tile is computed (16 KiB per wavefront in flight).
// NCK: 64-rank chunks of r_k per wavefront (r_k <= 512 NCK); NVT: 32-rank tiles of r_v per wavefront (r_v <= 256 NVT).
// Output per (sequence, part): the running maximum m and sum l per head, and U / l in fp16, [r_v][32 heads].
// ---------------------------------------------------------------------------------------------------------------
template <int NCK, int NVT>
__global__ void __launch_bounds__(512, 1) decode_core_kernel(DecodeCoreArgs a) {
  __shared__ __attribute__((aligned(16))) h8 wlds[NCK * 8 * 4][64];      // absorbed queries, fragment-major
  __shared__ __attribute__((aligned(16))) f4v sx[2][8][4][64];           // partial score tiles [parity][wavefront][quad][lane]

  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // this workgroup's (sequence, part): slot blockIdx.x of the balanced split (a workgroup past the last slot has nothing to do)
  int b, sp, nparts;
  {
    int parts, first;
    decode_parts_of_lane(a.n_keys, a.B, a.t_max, a.nsplit, lane, parts, first);
    if (a.B > 64) {
      b = blockIdx.x / a.nsplit;
      sp = blockIdx.x % a.nsplit;
      nparts = a.nsplit;
    } else {
      const unsigned long long mine = __ballot((int)blockIdx.x >= first && (int)blockIdx.x < first + parts);
      if (mine == 0) return;              // the same in every wavefront: the whole workgroup leaves
      b = __builtin_ctzll(mine);
      sp = (int)blockIdx.x - __shfl(first, b, 64);
      nparts = __shfl(parts, b, 64);
    }
    b = __builtin_amdgcn_readfirstlane(b);
    sp = __builtin_amdgcn_readfirstlane(sp);
    nparts = __builtin_amdgcn_readfirstlane(nparts);
  }
  const int kch = (a.r_k + 63) / 64, vtl = (a.r_v + 31) / 32, ktiles = (a.t_max + 31) / 32;
  int n = a.n_keys[b];
  n = n < 0 ? 0 : (n > a.t_max ? a.t_max : n);
  const int ntiles = (n + 31) / 32;
  const int tps = (ntiles + nparts - 1) / nparts;
  const int j0 = sp * tps, j1 = (j0 + tps < ntiles) ? j0 + tps : ntiles;

  float m_run = -1e30f, l_run = 0.f;
  f16v u[NVT];
#pragma unroll
  for (int i = 0; i < NVT; ++i) u[i] = zero16();

  if (j0 < j1) {
    const long long k_total = (long long)fm_bytes(a.t_max, a.r_k);
    const long long v_total = (long long)vtl * ktiles * 2048;
    const char* kbase = (const char*)a.kcache + (size_t)b * k_total;
    const char* vbase = (const char*)a.vcache + (size_t)b * v_total;
    h8 kf[NCK][4], vf[NVT][2], kn[NCK][4], vn[NVT][2];
    auto request = [&](int j, h8 (&kd)[NCK][4], h8 (&vd)[NVT][2]) {
#pragma unroll
      for (int i = 0; i < NCK; ++i) {
        const int c = wave + 8 * i;                       // chunks past r_k: resource of size 0 -> zeros
        const rsrc_t r = rsrc_at(kbase, c < kch ? k_total : 0, ((long long)j * kch + c) * kFmChunkBytes);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) kd[i][kk] = __builtin_bit_cast(h8, buf_load16(r, kk * kFmStepBytes + lane * 16));
      }
#pragma unroll
      for (int i = 0; i < NVT; ++i) {
        const int rt = wave + 8 * i;
        const rsrc_t r = rsrc_at(vbase, rt < vtl ? v_total : 0, ((long long)j * vtl + rt) * 2048);
#pragma unroll
        for (int s = 0; s < 2; ++s) vd[i][s] = __builtin_bit_cast(h8, buf_load16(r, s * 1024 + lane * 16));
      }
    };
    request(j0, kf, vf);
    // absorbed queries of this sequence -> LDS (fragment-major bytes as they lie), while the first tile is in flight
    {
      const u4* src = (const u4*)((const char*)a.W + (size_t)b * kch * 4096);
      for (int i = tid; i < kch * 256; i += 512) ((u4*)wlds)[i] = src[i];
    }
    __syncthreads();
    int par = 0;
    // one key tile: operands kc / vc of tile j are in registers, those of tile j + 1 are requested into kx / vx and are
    // first touched in the next call (the two register sets swap roles instead of being copied, so nothing waits for a
    // load before its first real use)
    auto tile_step = [&](int j, h8 (&kc)[NCK][4], h8 (&vc)[NVT][2], h8 (&kx)[NCK][4], h8 (&vx)[NVT][2]) {
      request(j + 1 < j1 ? j + 1 : j, kx, vx);            // the last tile is requested twice; nothing is read out of range
      // ---- partial scores of this wavefront's rank chunks
      f16v sp_ = zero16();
#pragma unroll
      for (int i = 0; i < NCK; ++i)
        if (wave + 8 * i < kch) {                          // wave-uniform; LDS past the last chunk was never written
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) sp_ = mfma32(kc[i][kk], wlds[(wave + 8 * i) * 4 + kk][lane], sp_);   // rows keys, cols heads
        }
#pragma unroll
      for (int qd = 0; qd < 4; ++qd) {
        f4v t;
#pragma unroll
        for (int e = 0; e < 4; ++e) t[e] = sp_[4 * qd + e];
        sx[par][wave][qd][lane] = t;
      }
      __syncthreads();
      f16v s = zero16();
#pragma unroll
      for (int w2 = 0; w2 < 8; ++w2)                       // the same order in every wavefront: identical sums
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
          const f4v t = sx[par][w2][qd][lane];
#pragma unroll
          for (int e = 0; e < 4; ++e) s[4 * qd + e] += t[e];
        }
      par ^= 1;
      // ---- mask, streaming softmax (log2 domain; W carries scale * log2 e)
      const int key0 = 32 * j;
      if (key0 + 32 > n) {
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (key0 + 8 * (v >> 2) + 4 * g + (v & 3) >= n) s[v] = -INFINITY;
      }
      float mx = s[0];
#pragma unroll
      for (int v = 1; v < 16; ++v) mx = fmaxf(mx, s[v]);
      mx = halves_max(mx);
      if (__any(mx > m_run + 8.0f)) {                      // lazily raised reference maximum, as in the prefill kernel
        const float m_new = fmaxf(m_run, mx);
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int i = 0; i < NVT; ++i)
#pragma unroll
          for (int v = 0; v < 16; ++v) u[i][v] *= alpha;
      }
      float sum = 0.f;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float p = __builtin_amdgcn_exp2f(s[v] - m_run);
        s[v] = p;
        sum += p;
      }
      l_run += sum;
      h8 pf[2];
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int e = 0; e < 8; ++e) pf[t][e] = (_Float16)s[8 * t + e];
      // ---- U^T += P_v^T tile x A^T for this wavefront's rank tiles
#pragma unroll
      for (int i = 0; i < NVT; ++i)
#pragma unroll
        for (int t = 0; t < 2; ++t) u[i] = mfma32(vc[i][t], pf[t], u[i]);   // rows ranks, cols heads
    };
    for (int j = j0; j < j1; j += 2) {
      tile_step(j, kf, vf, kn, vn);
      if (j + 1 < j1) tile_step(j + 1, kn, vn, kf, vf);
    }
  }

  // ---- partial results of this part
  const float l_tot = halves_sum(l_run);
  const size_t slot = blockIdx.x;          // = first slot of the sequence + part
  if (wave == 0 && g == 0) {
    a.stats[slot * 64 + l32] = m_run;
    a.stats[slot * 64 + 32 + l32] = l_tot;
  }
  if (j0 < j1) {
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    _Float16* up = a.upart + slot * (size_t)a.r_v * 32;
#pragma unroll
    for (int i = 0; i < NVT; ++i) {
      const int rt = wave + 8 * i;
      if (rt < vtl) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int rank = 32 * rt + 8 * (v >> 2) + 4 * g + (v & 3);
          if (rank < a.r_v) up[(size_t)rank * 32 + l32] = (_Float16)(u[i][v] * inv);
        }
      }
    }
  }
}

// merge the parts of one sequence: u[b, h, :] = sum_s wgt_s U_s / sum_s wgt_s, wgt_s = l_s 2^(m_s - max m).
// One workgroup per (64 ranks, sequence): the partial sums are read as they were written (32 heads contiguous per rank,
// 16 bytes = 8 heads per lane; the first 16 parts are requested before the weights are worked out, so the two waits
// overlap), transposed through LDS and written as runs of 64 ranks per head.
__global__ void __launch_bounds__(256) decode_merge_kernel(const float* __restrict__ stats, const _Float16* __restrict__ upart,
                                                           const int32_t* __restrict__ n_keys, int B, int t_max, int nsplit, int H,
                                                           int r_v, float* u_out) {
  __shared__ float tile[32][65];
  __shared__ float wgt[32][32];               // [part][head], normalised weights
  __shared__ float st[32][64];                // the parts' statistics
  const int r0 = 64 * blockIdx.x, b = blockIdx.y;
  int np, first_slot;
  {
    int parts, first;
    decode_parts_of_lane(n_keys, B, t_max, nsplit, threadIdx.x & 63, parts, first);
    np = B > 64 ? nsplit : __shfl(parts, b, 64);
    first_slot = B > 64 ? b * nsplit : __shfl(first, b, 64);
    np = __builtin_amdgcn_readfirstlane(np);
    first_slot = __builtin_amdgcn_readfirstlane(first_slot);
  }
  const size_t slot0 = (size_t)first_slot;
  // thread -> (rank rl, 8 heads from h0)
  const int rl = threadIdx.x >> 2, h0 = 8 * (threadIdx.x & 3), rho = r0 + rl;
  h8 x[16];
#pragma unroll
  for (int s = 0; s < 16; ++s) {
    x[s] = h8{};
    if (s < np && rho < r_v) x[s] = *(const h8*)&upart[((slot0 + s) * r_v + rho) * 32 + h0];
  }
  for (int i = threadIdx.x; i < np * 64; i += 256) st[i >> 6][i & 63] = stats[slot0 * 64 + i];
  __syncthreads();
  if (threadIdx.x < 32) {
    const int h = threadIdx.x;
    float M = -1e30f;
    for (int s = 0; s < np; ++s)
      if (st[s][32 + h] > 0.f) M = fmaxf(M, st[s][h]);
    float tot = 0.f;
    for (int s = 0; s < np; ++s) {
      const float l = st[s][32 + h];
      const float w = l > 0.f ? l * exp2f(st[s][h] - M) : 0.f;
      wgt[s][h] = w;
      tot += w;
    }
    const float inv = tot > 0.f ? 1.0f / tot : 0.f;
    for (int s = 0; s < np; ++s) wgt[s][h] *= inv;
  }
  __syncthreads();
  {
    // fixed order.  A part without keys has weight 0 and whatever its slot holds is discarded by the select, not multiplied.
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
#pragma unroll
    for (int s = 0; s < 16; ++s) {
      if (s < np) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float w = wgt[s][h0 + e];
          acc[e] += w > 0.f ? w * (float)x[s][e] : 0.f;
        }
      }
    }
    for (int s = 16; s < np; ++s) {
      h8 y = {};
      if (rho < r_v) y = *(const h8*)&upart[((slot0 + s) * r_v + rho) * 32 + h0];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float w = wgt[s][h0 + e];
        acc[e] += w > 0.f ? w * (float)y[e] : 0.f;
      }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) tile[h0 + e][rl] = acc[e];
  }
  __syncthreads();
  const int rl2 = threadIdx.x & 63;
  for (int k = 0; k < 8; ++k) {
    const int hh = (threadIdx.x >> 6) + 4 * k;
    if (hh < H && r0 + rl2 < r_v) u_out[((size_t)b * H + hh) * r_v + r0 + rl2] = tile[hh][rl2];
  }
}

// context[b, h d_h + d] = sum_rho u[b, h, rho] V_v[rho, h d_h + d] + b_v[h d_h + d], fp16 row-major [B, D].
// One workgroup per (head, 32 columns), on the matrix cores as ctx^T [columns, sequences] = V_v[:, columns]^T u^T: the
// ranks are dealt to the four wavefronts in chunks of 64; a wavefront copies its [64, 32] piece of V_v into its own
// part of LDS (rows padded as for the other staged weight tiles) and reads it back with the transposing read, the
// u operands (rounded to fp16) come straight from memory.  The four partial tiles are added through LDS.
__global__ void __launch_bounds__(256) decode_value_kernel(const float* __restrict__ u, const void* __restrict__ Vv, const void* __restrict__ bv,
                                                           int w_dt, int B, int D, int H, int r_v, _Float16* ctx) {
  constexpr int WS = wtile_stride(32);          // halves per staged row
  __shared__ __attribute__((aligned(16))) _Float16 vt[4][64 * WS];
  __shared__ float red[4][16][64];
  const int dh = D / H, h = blockIdx.x, col0 = h * dh + 32 * blockIdx.y;
  const int lane = threadIdx.x & 63, l32 = lane & 31, g = lane >> 5, wave = threadIdx.x >> 6;
  const int nch = (r_v + 63) / 64;
  const int tr = tr_lane_off(lane, WS) + 8 * g * WS;
  _Float16* mine = &vt[wave][0];
  for (int b0 = 0; b0 < B; b0 += 32) {
    const int b = b0 + l32;
    f16v acc = zero16();
    for (int ch = wave; ch < nch; ch += 4) {
      // rows 64 ch .., 32 columns: lane -> row lane / 4 (+ 16 per pass), 8 columns from 8 (lane % 4)
#pragma unroll
      for (int pss = 0; pss < 4; ++pss) {
        const int row = 16 * pss + (lane >> 2), rho = 64 * ch + row;
        u4 raw = {0u, 0u, 0u, 0u};
        if (rho < r_v) raw = *(const u4*)((const uint16_t*)Vv + (size_t)rho * D + col0 + 8 * (lane & 3));
        if (w_dt == DT_BF16) stage_store16<DT_BF16>(mine + row * WS + 8 * (lane & 3), raw);
        else stage_store16<DT_F16>(mine + row * WS + 8 * (lane & 3), raw);
      }
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const int rho = 64 * ch + 16 * s + 8 * g;
        h8 uf = {0, 0, 0, 0, 0, 0, 0, 0};
        if (b < B && rho < r_v) {
          const f4v* up = (const f4v*)(u + ((size_t)b * H + h) * r_v + rho);
          const f4v lo = up[0], hi = up[1];
#pragma unroll
          for (int i = 0; i < 4; ++i) { uf[i] = (_Float16)lo[i]; uf[4 + i] = (_Float16)hi[i]; }
        }
        const h8 vf = tr_frag(mine + tr + 16 * s * WS, mine + tr + (16 * s + 4) * WS);
        acc = mfma32(vf, uf, acc);
      }
    }
    __syncthreads();                             // the previous sequence tile's sums have been read
#pragma unroll
    for (int v = 0; v < 16; ++v) red[wave][v][lane] = acc[v];
    __syncthreads();
    if (wave == 0 && b < B) {
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const int d = 8 * jj + 4 * g;
        h4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int v = 4 * jj + e;
          const float sum = red[0][v][lane] + red[1][v][lane] + red[2][v][lane] + red[3][v][lane];
          o[e] = (_Float16)(sum + (bv ? load_param(bv, (size_t)col0 + d + e, w_dt) : 0.f));
        }
        *(h4*)(ctx + (size_t)b * D + col0 + d) = o;
      }
    }
  }
}

// The step's own bookkeeping in one launch: the new token's rows pk [B, r_k], pv [B, r_v] go to position t_len[b] of the
// two caches (same addressing as decode_cache_write_kernel) and n_keys[b] = t_len[b] + 1 (the new token is part of its
// own context).  One thread per 16-byte unit of pk, then one per element of pv.
__global__ void __launch_bounds__(256) decode_append_kernel(const _Float16* __restrict__ pk, const _Float16* __restrict__ pv,
                                                            const int32_t* __restrict__ t_len, int B, int t_max, int r_k, int r_v,
                                                            _Float16* kcache, _Float16* vcache, size_t k_seq_halves, size_t v_seq_halves,
                                                            int32_t* n_keys) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  const int per_seq = r_k / 8 + r_v;
  if (i >= B * per_seq) return;
  const int b = i / per_seq, j = i % per_seq;
  const int t = t_len[b];
  if (j == 0) n_keys[b] = t + 1;
  if (t < 0 || t >= t_max) return;
  if (j < r_k / 8) {
    const int rho = 8 * j, kch = (r_k + 63) / 64, off = rho & 63;
    const size_t unit = ((size_t)((t >> 5) * kch + (rho >> 6)) * 4 + ((off >> 3) & 3)) * 64 + (off >> 5) * 32 + (t & 31);
    *(h8*)(kcache + b * k_seq_halves + unit * 8) = *(const h8*)(pk + (size_t)b * r_k + rho);
  } else {
    const int rho = j - r_k / 8, vtl = (r_v + 31) / 32, kq = t & 31, o = kq & 15;
    const size_t unit = ((size_t)((t >> 5) * vtl + (rho >> 5)) * 2 + (kq >> 4)) * 64 + ((o >> 2) & 1) * 32 + (rho & 31);
    vcache[b * v_seq_halves + unit * 8 + (o & 3) + 4 * (o >> 3)] = pv[(size_t)b * r_v + rho];
  }
}

}  // namespace

hipError_t launch_decode_cache_write(const void* src, const int32_t* t_start, int B, int t_max, int r, int n_new, int which,
                                     void* cache, hipStream_t s) {
  const size_t seq_halves = (which == 0 ? fm_bytes(t_max, r) : decode_vcache_seq_bytes(t_max, r)) / 2;
  const size_t total = which == 0 ? (size_t)B * n_new * (r / 8) : (size_t)B * n_new * r;
  hipLaunchKernelGGL(decode_cache_write_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const _Float16*)src, t_start,
                     B, t_max, r, n_new, which, (_Float16*)cache, seq_halves, total);
  return hipGetLastError();
}

hipError_t launch_decode_absorb(const void* q, const void* Vk, int w_dt, int B, int D, int H, int r_k, float scale, void* W,
                                hipStream_t s) {
  hipLaunchKernelGGL(decode_absorb_kernel, dim3((r_k + 63) / 64, H), dim3(256), 0, s, (const _Float16*)q, Vk, w_dt, B, D, H, r_k,
                     scale * kLog2eD, (_Float16*)W);
  return hipGetLastError();
}

hipError_t launch_decode_core(const DecodeCoreArgs& a, hipStream_t s) {
  const dim3 grid(a.B * a.nsplit), block(512);
  const int nck = ((a.r_k + 63) / 64 + 7) / 8, nvt = ((a.r_v + 31) / 32 + 7) / 8;
  if (nck > 2 || nvt > 4) return hipErrorInvalidValue;
  if (nck <= 1 && nvt <= 1) hipLaunchKernelGGL((decode_core_kernel<1, 1>), grid, block, 0, s, a);
  else if (nck <= 1 && nvt <= 2) hipLaunchKernelGGL((decode_core_kernel<1, 2>), grid, block, 0, s, a);
  else if (nvt <= 2) hipLaunchKernelGGL((decode_core_kernel<2, 2>), grid, block, 0, s, a);
  else hipLaunchKernelGGL((decode_core_kernel<2, 4>), grid, block, 0, s, a);
  return hipGetLastError();
}

hipError_t launch_decode_merge(const float* stats, const void* upart, const int32_t* n_keys, int B, int t_max, int nsplit, int H, int r_v,
                               float* u_out, hipStream_t s) {
  hipLaunchKernelGGL(decode_merge_kernel, dim3((r_v + 63) / 64, B), dim3(256), 0, s, stats, (const _Float16*)upart, n_keys, B, t_max, nsplit,
                     H, r_v, u_out);
  return hipGetLastError();
}

hipError_t launch_decode_value(const float* u, const void* Vv, const void* bv, int w_dt, int B, int D, int H, int r_v, void* ctx,
                               hipStream_t s) {
  hipLaunchKernelGGL(decode_value_kernel, dim3(H, (D / H) / 32), dim3(256), 0, s, u, Vv, bv, w_dt, B, D, H, r_v, (_Float16*)ctx);
  return hipGetLastError();
}

hipError_t launch_decode_append(const void* pk, const void* pv, const int32_t* t_len, int B, int t_max, int r_k, int r_v,
                                void* kcache, void* vcache, int32_t* n_keys, hipStream_t s) {
  const int total = B * (r_k / 8 + r_v);
  hipLaunchKernelGGL(decode_append_kernel, dim3((total + 255) / 256), dim3(256), 0, s, (const _Float16*)pk, (const _Float16*)pv, t_len,
                     B, t_max, r_k, r_v, (_Float16*)kcache, (_Float16*)vcache, fm_bytes(t_max, r_k) / 2,
                     decode_vcache_seq_bytes(t_max, r_v) / 2, n_keys);
  return hipGetLastError();
}

}  // namespace fsvd
