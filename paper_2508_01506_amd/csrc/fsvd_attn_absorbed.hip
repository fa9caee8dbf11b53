// Streaming attention for per-head factors of rank r <= 64 in the "absorbed" schedule (Alg. 1 in its own per-head
// setting, V_a in r x d_h; appendix on multi-head low-rank activations): no Q, K or V tile is ever rebuilt, every
// product of the loop contracts over a rank axis.
//   M_h   = V_q^h (V_k^h)^T                      [r_q, r_k]       once per workgroup (a few matrix-core steps)
//   w_h   = scale * (P_q^h M_h + b_q^h (V_k^h)^T) [queries, r_k]  = scale * q_h (V_k^h)^T: the key projection absorbed
//                                                                 into the queries; the term q_h . b_k is the same for
//                                                                 every key of a row and cancels in the softmax
//   S     = w_h (P_k^h)^T                        [queries, keys]  contraction over r_k instead of d_h
//   u_h   = sum_j alpha_j P_v^h[j] / l           [queries, r_v]   streaming softmax, accumulated in rank space
//   ctx_h = u_h V_v^h + b_v^h                                     the value projection applied once, at the end; the
//                                                                 weights alpha sum to one, so b_v passes through
// P_a^h are columns [h r_a, (h+1) r_a) of the concatenated rank axis of P_a [T, H r_a] (fragment-major).
//
// One workgroup (4 wavefronts) owns one (sequence, head, block of 128 queries); every wavefront owns 32 queries.  All
// products are transposed (keys / ranks / features along accumulator rows, queries along lanes), so that an accumulator
// is the next product's operand without leaving its registers.  A fragment-major 16-byte unit holds 8 consecutive ranks
// of one token: to make such a unit one operand register set, rows and columns of M_h are computed in a permuted order
// (sigma below), after which the accumulator rows of w_h come out in exactly the order of P_k's units.  P_q and P_k
// operands are therefore loaded straight from memory; only P_v (needed with keys as the contraction index) and V_v
// (needed transposed) go through LDS and its transposing read.
#include "fsvd_common.h"
#include "fsvd_kernels.h"

namespace fsvd {

namespace {

constexpr int kAbsWaves = 4;
constexpr int kAbsThreads = kAbsWaves * 64;
constexpr int kAbsBQ = kAbsWaves * 32;       // queries per workgroup
constexpr int kAbsBKV = 128;                 // keys per step
constexpr float kLog2eA = 1.4426950408889634f;

// byte offset of the 16-byte unit (token, octet o of the contraction axis) of a fragment-major tensor with kchunks chunks
__device__ __forceinline__ int fm_unit_off(int tok, int kchunks, int o) {
  return ((tok >> 5) * kchunks + (o >> 3)) * kFmChunkBytes + (o & 3) * kFmStepBytes + ((((o >> 2) & 1) << 5) + (tok & 31)) * 16;
}
// KS: matrix-core steps of 16 ranks that cover the largest of r_q, r_k, r_v (1..4); smaller ranks leave zero operands
// wavefronts per SIMD the register budget is set for (= workgroups per compute unit): what the LDS tiles leave room for
constexpr int abs_occupancy(int DH, int KS) { return KS <= 2 ? 4 : ((DH == 128 && KS == 4) ? 2 : 3); }

template <int DH, int WT, int KS>
__global__ void __launch_bounds__(kAbsThreads, abs_occupancy(DH, KS)) attn_absorbed_kernel(AttnCoreArgs a, int nqb) {
  constexpr int DT32 = DH / 32, DST = DH / 16;
  constexpr int NT = (KS + 1) / 2;                       // 32-rank tiles
  constexpr int WS = wtile_stride(DH);
  constexpr int PVS = NT == 1 ? 32 : wtile_stride(64);   // halves per row of the P_v tile: 64-byte rows need no padding
  constexpr int OB = NT == 1 ? 2 : 3;                    // log2 of the octets staged per key of P_v
  constexpr int NJV = (kAbsBKV << OB) / kAbsThreads;     // P_v units per thread and step
  constexpr int NJK = kAbsBKV * 2 * KS / kAbsThreads;    // P_k units per thread and step (= KS)

  __shared__ __attribute__((aligned(16))) _Float16 wv[16 * KS * WS];               // V_v^h [rank][DH], zero rows from r_v on
  __shared__ __attribute__((aligned(16))) _Float16 pv[kAbsBKV * PVS];              // P_v^h [key][rank], zero columns from r_v on
  __shared__ __attribute__((aligned(16))) u4 pk[4][KS][64];                        // P_k^h operands [key tile][step][lane]

  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int BH = a.B * a.H;
  const int bh = blockIdx.x % BH;
  const int qb = nqb - 1 - blockIdx.x / BH;   // late query blocks (most keys under a causal mask) first
  const int b = bh / a.H, h = bh % a.H;
  const int M = a.M, D = a.D, T = a.B * a.M;
  const int q0 = qb * kAbsBQ, qw = q0 + wave * 32;
  int kv_len = a.key_len ? a.key_len[b] : M;
  kv_len = kv_len < 1 ? 1 : (kv_len > M ? M : kv_len);
  int kv_end = kv_len;
  if (a.causal && q0 + kAbsBQ < kv_end) kv_end = q0 + kAbsBQ;
  const int nsteps = (kv_end + kAbsBKV - 1) / kAbsBKV;
  const int tok0 = b * M, col0 = h * DH;
  const int rq = a.rq, rk = a.rk, rv = a.rv;
  const int pch_q = (a.H * rq + kChunkK - 1) / kChunkK, pch_k = (a.H * rk + kChunkK - 1) / kChunkK,
            pch_v = (a.H * rv + kChunkK - 1) / kChunkK;
  const rsrc_t rsPq = rsrc_at(a.Pq, (long long)fm_bytes(T, a.H * rq), 0);
  const rsrc_t rsPk = rsrc_at(a.Pk, (long long)fm_bytes(T, a.H * rk), 0);
  const rsrc_t rsPv = rsrc_at(a.Pv, (long long)fm_bytes(T, a.H * rv), 0);
  const int oq0 = (h * rq) >> 3, ok0 = (h * rk) >> 3, ov0 = (h * rv) >> 3;        // first octet of the head's rank windows

  // ---- staging of one step of 128 keys.  P_v: unit u = tid + 256 j -> (key u >> OB, octet u % 2^OB), written as rows
  // [key][rank].  P_k: unit u -> (key tile, matrix-core step s, lane) in operand order: lane (key, g) of step s holds
  // octet 2 s + g of the head's window.  Octets from the rank on are zeros.
  u4 v_raw[NJV], k_raw[NJK];
  auto issue_kv = [&](int step) {
#pragma unroll
    for (int j = 0; j < NJV; ++j) {
      const int u = tid + kAbsThreads * j, oct = u & ((1 << OB) - 1);
      int key = step * kAbsBKV + (u >> OB);
      key = key < M ? key : M - 1;
      v_raw[j] = buf_load16(rsPv, 8 * oct < rv ? fm_unit_off(tok0 + key, pch_v, ov0 + oct) : kOobOffset);
    }
#pragma unroll
    for (int j = 0; j < NJK; ++j) {
      const int u = tid + kAbsThreads * j, ln = u & 63, st = (u >> 6) % KS, kt = (u >> 6) / KS, oct = 2 * st + (ln >> 5);
      int key = step * kAbsBKV + 32 * kt + (ln & 31);
      key = key < M ? key : M - 1;
      k_raw[j] = buf_load16(rsPk, 8 * oct < rk ? fm_unit_off(tok0 + key, pch_k, ok0 + oct) : kOobOffset);
    }
  };
  auto commit_kv = [&]() {
#pragma unroll
    for (int j = 0; j < NJV; ++j) {
      const int u = tid + kAbsThreads * j, oct = u & ((1 << OB) - 1);
      *(u4*)&pv[(u >> OB) * PVS + 8 * oct] = v_raw[j];
    }
#pragma unroll
    for (int j = 0; j < NJK; ++j) (&pk[0][0][0])[tid + kAbsThreads * j] = k_raw[j];
  };

  issue_kv(0);
  u4 pq_raw[KS];
  {
    int q = qw + l32;
    q = q < M ? q : M - 1;
#pragma unroll
    for (int s = 0; s < KS; ++s)
      pq_raw[s] = buf_load16(rsPq, 16 * s + 8 * g < rq ? fm_unit_off(tok0 + q, pch_q, oq0 + 2 * s + g) : kOobOffset);
  }
  // ---- V_v^h -> LDS as it lies in memory (16 bytes per lane); rows from r_v on are zeros
  {
    constexpr int LPR = DH / 8, NU = (16 * KS * LPR + kAbsThreads - 1) / kAbsThreads;
    const rsrc_t rs = rsrc_at(a.Vv, (long long)a.H * rv * DH * 2, 0);
#pragma unroll
    for (int j = 0; j < NU; ++j) {
      const int u = tid + kAbsThreads * j, row = u / LPR, c8 = 8 * (u % LPR);
      if (row < 16 * KS) {
        const u4 raw = buf_load16(rs, row < rv ? ((h * rv + row) * DH + c8) * 2 : kOobOffset);
        stage_store16<WT>(&wv[row * WS + c8], raw);
      }
    }
  }

  // =================================== absorbed queries: W^T [r_k, 32 queries] ===================================
  // Row / column c of a 32-rank tile of M_h stands for rank 32 tile + sigma(c), sigma = c with bits 2 and 3 swapped:
  // accumulator register v of lane group g is row 8 (v / 4) + 4 g + v % 4, so registers 8 t .. 8 t + 7 are then the 8
  // consecutive ranks 16 t + 8 g .. of the tile: one fragment-major unit of P_q (for M_h's rows) or P_k (for W's rows).
  // M_h is the same for the whole workgroup: its 32 x 32 tiles are dealt to the wavefronts (tile (tq, tk) to wavefront
  // 2 tq + tk, so that not every wavefront of every workgroup asks the L2 for the same few lines of V_q and V_k at the
  // same moment), handed over through LDS as ready operands, and every wavefront multiplies them with its own queries.
  h8 wq[KS];
  {
    constexpr int DSB = DST < 4 ? DST : 4;     // contraction steps whose operands are requested together
    u4* const mfl = (u4*)pv;                   // [tk][step s][lane]: M_h operands (the P_v tile is not in use yet)
    f4v* const wbl = (f4v*)(mfl + NT * KS * 64);   // [tk][quad][lane]: b_q (V_k^h)^T, rows r_k, the same in every column
    static_assert(NT * KS * 64 * 16 + NT * 4 * 64 * 16 <= kAbsBKV * PVS * 2, "the hand-over must fit in the P_v tile");
    const float qs = a.scale * kLog2eA;
    const int tq = wave >> 1, tk = wave & 1;
    if (tq < NT && tk < NT) {
      const int sig = (l32 & ~12) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);
      const rsrc_t rsVq = rsrc_at(a.Vq, (long long)a.H * rq * DH * 2, 0);
      const rsrc_t rsVk = rsrc_at(a.Vk, (long long)a.H * rk * DH * 2, 0);
      const rsrc_t rsBq = rsrc_at(a.bq, a.bq ? (long long)D * 2 : 0, 0);
      const int rowq = 32 * tq + sig, rowk = 32 * tk + sig;
      f16v macc = zero16(), bacc = zero16();
#pragma unroll
      for (int d0 = 0; d0 < DST; d0 += DSB) {
        u4 vq_raw[DSB], vk_raw[DSB], bq_raw[DSB];
#pragma unroll
        for (int ds = 0; ds < DSB; ++ds) {
          const int dof = (16 * (d0 + ds) + 8 * g) * 2;
          vk_raw[ds] = buf_load16(rsVk, rowk < rk ? (h * rk + rowk) * DH * 2 + dof : kOobOffset);
          vq_raw[ds] = buf_load16(rsVq, rowq < rq ? (h * rq + rowq) * DH * 2 + dof : kOobOffset);
          bq_raw[ds] = buf_load16(rsBq, tq == 0 ? col0 * 2 + dof : kOobOffset);      // zeros without a bias
        }
#pragma unroll
        for (int ds = 0; ds < DSB; ++ds) {
          const h8 vk = raw_to_h8<WT>(vk_raw[ds]);
          macc = mfma32(raw_to_h8<WT>(vq_raw[ds]), vk, macc);                        // rows r_q, cols r_k
          if (tq == 0) bacc = mfma32(vk, raw_to_h8<WT>(bq_raw[ds]), bacc);           // rows r_k, every column the same
        }
      }
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        if (2 * tq + t < KS) {
          h8 mf;
#pragma unroll
          for (int i = 0; i < 8; ++i) mf[i] = (_Float16)macc[8 * t + i];
          mfl[(tk * KS + 2 * tq + t) * 64 + lane] = __builtin_bit_cast(u4, mf);
        }
      }
      if (tq == 0) {
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
          f4v x;
#pragma unroll
          for (int e = 0; e < 4; ++e) x[e] = bacc[4 * qd + e];
          wbl[(tk * 4 + qd) * 64 + lane] = x;
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int tk2 = 0; tk2 < NT; ++tk2) {
      f16v wacc;
#pragma unroll
      for (int qd = 0; qd < 4; ++qd) {
        const f4v x = wbl[(tk2 * 4 + qd) * 64 + lane];
#pragma unroll
        for (int e = 0; e < 4; ++e) wacc[4 * qd + e] = x[e];
      }
#pragma unroll
      for (int s = 0; s < KS; ++s)
        wacc = mfma32(__builtin_bit_cast(h8, mfl[(tk2 * KS + s) * 64 + lane]), __builtin_bit_cast(h8, pq_raw[s]), wacc);   // rows r_k, cols queries
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        if (2 * tk2 + t < KS) {
          h8 r;
#pragma unroll
          for (int i = 0; i < 8; ++i) r[i] = (_Float16)(wacc[8 * t + i] * qs);
          wq[2 * tk2 + t] = r;
        }
      }
    }
  }

  // =================================== key / value loop ===================================
  const int trV = tr_lane_off(lane, PVS) + 4 * g * PVS;
  f16v u[NT];
#pragma unroll
  for (int i = 0; i < NT; ++i) u[i] = zero16();
  float m_run = 0.f, l_run = 0.f;
  bool first = true;
  h8 kone = {}, qneg;
  kone[0] = g == 0 ? (_Float16)1.0f : (_Float16)0.0f;
  kone[1] = kone[0];
  auto set_qneg = [&]() {      // -m_run as an fp16 head + tail in two contraction slots: the matrix core subtracts the reference
    const _Float16 hi = (_Float16)(-m_run);
    const _Float16 lo = (_Float16)(-m_run - (float)hi);
    qneg = h8{};
    qneg[0] = g == 0 ? hi : (_Float16)0.0f;
    qneg[1] = g == 0 ? lo : (_Float16)0.0f;
  };
  set_qneg();
  const int qlast = qw + 31;

  for (int step = 0; step < nsteps; ++step) {
    __syncthreads();                 // every wavefront is done with the previous step's tiles
    commit_kv();
    if (step + 1 < nsteps) issue_kv(step + 1);
    __syncthreads();
#pragma unroll 1
    for (int ks = 0; ks < 4; ++ks) {
      const int key0 = step * kAbsBKV + 32 * ks;
      if (key0 >= kv_end) break;
      if (a.causal && key0 > qlast) break;
      f16v s = mfma32(kone, qneg, zero16());
#pragma unroll
      for (int i = 0; i < KS; ++i) s = mfma32(__builtin_bit_cast(h8, pk[ks][i][lane]), wq[i], s);   // S^T - m: rows keys, cols queries
      const bool need_mask = (key0 + 32 > kv_len) || (a.causal && key0 + 31 > qw);
      if (need_mask) {
        const int q = qw + l32;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = key0 + 8 * (v >> 2) + 4 * g + (v & 3);
          if (key >= kv_len || (a.causal && key > q)) s[v] = -INFINITY;
        }
      }
      // lazily raised reference maximum in the log2 domain, as in the rebuilding kernel
      float mx = s[0];
#pragma unroll
      for (int v = 1; v < 16; ++v) mx = fmaxf(mx, s[v]);
      mx = halves_max(mx);
      if (__any(first || mx > 8.0f)) {
        const float delta = first ? fmaxf(mx, -1e30f) : fmaxf(mx, 0.f);
        const float alpha = first ? 0.f : __builtin_amdgcn_exp2f(-delta);
        m_run += delta;
        l_run *= alpha;
        set_qneg();
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] -= delta;
#pragma unroll
        for (int i = 0; i < NT; ++i)
#pragma unroll
          for (int v = 0; v < 16; ++v) u[i][v] *= alpha;
      }
      first = false;
      float sum = 0.f;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float p = __builtin_amdgcn_exp2f(s[v]);
        s[v] = p;
        sum += p;
      }
      l_run += sum;
      h8 pf[2];
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int e = 0; e < 8; ++e) pf[t][e] = (_Float16)s[8 * t + e];
#pragma unroll
      for (int i = 0; i < NT; ++i) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const _Float16* vq = pv + (32 * ks + 16 * t) * PVS + trV + 32 * i;
          u[i] = mfma32(tr_frag(vq, vq + 8 * PVS), pf[t], u[i]);      // U^T: rows ranks, cols queries
        }
      }
    }
  }

  // =================================== value projection, once ===================================
  // ctx^T [DH, queries] = (V_v^h)^T U^T: the normalised accumulators are the operand as they are
  f16v o[DT32];
#pragma unroll
  for (int dt = 0; dt < DT32; ++dt) o[dt] = zero16();
  {
    const float l = halves_sum(l_run);
    const float inv = l > 0.f ? 1.0f / l : 0.f;
    const int trW = tr_lane_off(lane, WS) + 4 * g * WS;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      h8 uf;
#pragma unroll
      for (int i = 0; i < 8; ++i) uf[i] = (_Float16)(u[s >> 1][8 * (s & 1) + i] * inv);
#pragma unroll
      for (int dt = 0; dt < DT32; ++dt) {
        const _Float16* wp = wv + 16 * s * WS + trW + 32 * dt;
        o[dt] = mfma32(tr_frag(wp, wp + 8 * WS), uf, o[dt]);
      }
    }
  }

  // ---- + b_v, write the context fragment-major: 4 consecutive features per 8-byte store
  {
    _Float16* C = (_Float16*)a.C;
    const int cch = D / 64;
    const int q = qw + l32;
    const rsrc_t rsBv = rsrc_at(a.bv, a.bv ? (long long)D * 2 : 0, 0);
    if (q < M) {
      const int tok = tok0 + q;
#pragma unroll
      for (int dt = 0; dt < DT32; ++dt) {
        const int dabs = col0 + 32 * dt;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const f4v bias = raw_to_f4<WT>(buf_load8(rsBv, (dabs + 8 * jj + 4 * g) * 2));
          const size_t unit = ((size_t)((tok >> 5) * cch + (dabs >> 6)) * 4 + jj) * 64 + ((dabs >> 5) & 1) * 32 + (tok & 31);
          h4 r;
#pragma unroll
          for (int i = 0; i < 4; ++i) r[i] = (_Float16)(o[dt][4 * jj + i] + bias[i]);
          *(h4*)(C + unit * 8 + 4 * g) = r;
        }
      }
    }
  }
}

template <int DH, int KS>
hipError_t launch_abs(const AttnCoreArgs& a, hipStream_t s) {
  const int nqb = (a.M + kAbsBQ - 1) / kAbsBQ;
  const dim3 grid(a.B * a.H * nqb), block(kAbsThreads);
  if (a.w_dt == DT_F16) hipLaunchKernelGGL((attn_absorbed_kernel<DH, DT_F16, KS>), grid, block, 0, s, a, nqb);
  else hipLaunchKernelGGL((attn_absorbed_kernel<DH, DT_BF16, KS>), grid, block, 0, s, a, nqb);
  return hipGetLastError();
}
template <int DH>
hipError_t launch_abs_dh(const AttnCoreArgs& a, hipStream_t s) {
  const int rmax = a.rq > a.rk ? (a.rq > a.rv ? a.rq : a.rv) : (a.rk > a.rv ? a.rk : a.rv);
  switch ((rmax + 15) / 16) {
    case 1: return launch_abs<DH, 1>(a, s);
    case 2: return launch_abs<DH, 2>(a, s);
    case 3: return launch_abs<DH, 3>(a, s);
    default: return launch_abs<DH, 4>(a, s);
  }
}

}  // namespace

bool attn_absorbed_supported(const AttnCoreArgs& a) {
  const int dh = a.H > 0 ? a.D / a.H : 0;
  return a.per_head == 1 && !a.tiled && (dh == 64 || dh == 128) && a.rq <= 64 && a.rk <= 64 && a.rv <= 64 &&
         a.rq % 16 == 0 && a.rk % 16 == 0 && a.rv % 16 == 0;
}

hipError_t launch_attn_absorbed(const AttnCoreArgs& a, hipStream_t s) {
  if (!attn_absorbed_supported(a)) return hipErrorInvalidValue;
  return a.D / a.H == 64 ? launch_abs_dh<64>(a, s) : launch_abs_dh<128>(a, s);
}

}  // namespace fsvd
