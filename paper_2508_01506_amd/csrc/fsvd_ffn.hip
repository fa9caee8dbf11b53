// Fused FFN core (Alg. 2, the on-chip loops): Z[T, r2] = phi(P1[T, r1] V_1[r1, F] + b_1) U_2[F, r2].
// The hidden activation phi(...) [T, F] exists only as 128-wide slabs in registers / LDS.
//
// One workgroup (4 wavefronts) owns 128 (or 64) tokens and one slice of at most 512 output ranks; the
// accumulator Z^T [slice, 128 tokens] stays in registers for the whole sweep over F.  Per 128-wide
// chunk of F:
//   phase A  Y^T[128 f, 128 tok] = V_1[:, chunk]^T P1^T, contraction over r1 in 128-wide stages;
//            wavefront (wt, wr) computes features 64*wr.. for tokens 64*wt.. (P1 rows come straight
//            from global memory), adds b_1, applies phi, rounds to fp16 and hands the result to its
//            partner wavefront through LDS in MFMA operand order;
//   phase B  Z^T[128*s + 64*wr.., tokens 64*wt..] += U_2[chunk, :]^T Y^T, one 128-rank sub-stage s at a
//            time.
// Every weight tile (128 contraction rows x 128 output columns) is copied as it lies in memory into a
// double-buffered LDS tile and read back with the LDS's transposing read; tile i+1 is fetched from global
// memory while tile i is used.
// When r2 > 512 the slices are separate workgroups and phase A is recomputed per slice.
#include "fsvd_common.h"
#include "fsvd_kernels.h"

namespace fsvd {

namespace {

constexpr int kFfnBF = 128;                 // F chunk
constexpr int kTile = 128;                  // weight tile edge
constexpr int kTileRow = wtile_stride(kTile);   // halves per LDS tile row
constexpr int kMaxSlice = 512;

// exact-GELU via the Abramowitz-Stegun 7.1.26 rational approximation of erf (|error| <= 1.5e-7),
// written so that the negative tail does not cancel.
__device__ __forceinline__ float gelu_erf_f(float x) {
  const float z = fabsf(x) * 0.70710678118654752f;
  const float t = __frcp_rn(1.0f + 0.3275911f * z);
  const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
  const float tail = 0.5f * poly * __builtin_amdgcn_exp2f(-z * z * 1.4426950408889634f);   // 0.5 * erfc(|x|/sqrt2)
  return x >= 0.f ? x * (1.0f - tail) : x * tail;
}
__device__ __forceinline__ float gelu_tanh_f(float x) {
  const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
  return x * __frcp_rn(1.0f + __builtin_amdgcn_exp2f(-2.0f * u * 1.4426950408889634f));
}

template <int NS, int WT, int TG>
__global__ void __launch_bounds__(256, 1) ffn_core_kernel(FfnCoreArgs a, int nslices, int slice_w) {
  constexpr int WRN = 4 / TG;          // wavefronts sharing one 64-token group, splitting features / ranks
  constexpr int FT = 4 / WRN;          // 32-wide feature (phase A) and rank (phase B) tiles per wavefront
  constexpr int ROWS = 128 / WRN;      // rows of a 128-wide tile owned by one wavefront
  __shared__ __attribute__((aligned(16))) _Float16 wt_lds[2][kTile * kTileRow];
  __shared__ __attribute__((aligned(16))) h8 gtile[TG][4][2][2][64];   // [token group][f tile][t][token tile][lane]

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
  const int wt = wave / WRN, wr = wave % WRN;
  const int slice = blockIdx.x % nslices;
  const int tb = blockIdx.x / nslices;
  const int t0 = tb * (64 * TG);
  const int s0 = slice * slice_w;                               // first output rank of this slice
  const int r1 = a.r1, F = a.F, r2 = a.r2, T = a.T;
  const int s_end = (s0 + slice_w < r2) ? s0 + slice_w : r2;
  const int nA = (r1 + kTile - 1) / kTile;
  const int nchunks = (F + kFfnBF - 1) / kFfnBF;
  const int pch = (r1 + 63) / 64, zch = (r2 + 63) / 64;
  const long long p_total = (long long)fm_bytes(T, r1);
  const long long v1_total = (long long)r1 * F * 2, u2_total = (long long)F * r2 * 2;

  // ---- weight tile staging: thread -> tile row s_r (+ 16 per pass), 8 columns from s_c; rows are copied as they
  // lie in memory, the LDS transposes on the way out
  const int s_r = tid >> 4, s_c = 8 * (tid & 15);
  u4 w_raw[8];
  // kind 0: V_1 rows r of stage idx, columns f of chunk c.  kind 1: U_2 rows f of chunk c, columns s0 + 128*idx.
  auto issue_tile = [&](int kind, int c, int idx) {
    if (kind == 0) {
      const rsrc_t r = rsrc_at(a.V1, v1_total, ((long long)idx * kTile * F + c * kFfnBF) * 2);
      const bool ok = c * kFfnBF + s_c < F;
#pragma unroll
      for (int p = 0; p < 8; ++p) w_raw[p] = buf_load16(r, ok ? ((s_r + 16 * p) * F + s_c) * 2 : kOobOffset);
    } else {
      const int n0 = s0 + idx * kTile;
      const rsrc_t r = rsrc_at(a.U2, u2_total, ((long long)c * kFfnBF * r2 + n0) * 2);
      const bool ok = n0 + s_c < s_end;
#pragma unroll
      for (int p = 0; p < 8; ++p) w_raw[p] = buf_load16(r, ok ? ((s_r + 16 * p) * r2 + s_c) * 2 : kOobOffset);
    }
  };
  auto commit_tile = [&](int pb) {
#pragma unroll
    for (int p = 0; p < 8; ++p) stage_store16<WT>(&wt_lds[pb][(s_r + 16 * p) * kTileRow + s_c], w_raw[p]);
  };
  const int trA = tr_lane_off(lane, kTileRow) + 32 * g * kTileRow;   // phase A: k rows 32 g + 8 kk + 0..7
  const int trB = tr_lane_off(lane, kTileRow) + 4 * g * kTileRow;    // phase B: k rows 16 fs + 4 g + {0..3, 8..11}

  // ---- P1 operands of this wavefront's tokens (fragment-major: one contiguous 1 KiB load each)
  int voffP[2];
#pragma unroll
  for (int tt = 0; tt < 2; ++tt) {
    int tok = t0 + 64 * wt + 32 * tt + l32;
    tok = tok < T ? tok : T - 1;
    voffP[tt] = fm_voff(tok, pch, g);
  }
  h8 pfr[2][4];
  auto load_p = [&](int half, int kk) {   // half: 64-wide piece of r1 (the rank padding of an FM tensor holds zeros;
                                          // a half beyond the tensor falls outside the resource)
    const rsrc_t r = rsrc_at(a.P1, (half < pch) ? p_total : 0, (long long)half * kFmChunkBytes);
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) pfr[tt][kk] = __builtin_bit_cast(h8, buf_load16(r, voffP[tt] + kk * kFmStepBytes));
  };
  const int nhalf = 2 * nA;

  f16v z[NS][FT][2];
#pragma unroll
  for (int s = 0; s < NS; ++s)
#pragma unroll
    for (int rt = 0; rt < FT; ++rt) { z[s][rt][0] = zero16(); z[s][rt][1] = zero16(); }

  int parity = 0;
  issue_tile(0, 0, 0);
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) load_p(0, kk);
  commit_tile(0);
  __syncthreads();

  for (int c = 0; c < nchunks; ++c) {
    // ================= phase A =================
    f16v y[FT][2];
#pragma unroll
    for (int ft = 0; ft < FT; ++ft) { y[ft][0] = zero16(); y[ft][1] = zero16(); }
    for (int ra = 0; ra < nA; ++ra) {
      const bool lastA = ra + 1 == nA;
      if (!lastA) issue_tile(0, c, ra + 1); else issue_tile(1, c, 0);
      const _Float16* wb = wt_lds[parity];
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        const int half = 2 * ra + hh;
        int nh = half + 1;
        if (nh == nhalf) nh = 0;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          h8 wf[FT];
#pragma unroll
          for (int ft = 0; ft < FT; ++ft) {
            const _Float16* q = wb + trA + (64 * hh + 8 * kk) * kTileRow + ROWS * wr + 32 * ft;
            wf[ft] = tr_frag(q, q + 4 * kTileRow);
          }
#pragma unroll
          for (int ft = 0; ft < FT; ++ft)
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) y[ft][tt] = mfma32(wf[ft], pfr[tt][kk], y[ft][tt]);   // rows f, cols tokens
          load_p(nh, kk);                 // refill the operand registers just consumed
        }
      }
      if (lastA) {
        // bias, phi, fp16, publish in operand order for phase B
        const rsrc_t rB = rsrc_at(a.b1, a.b1 ? (long long)F * 2 : 0, (long long)c * kFfnBF * 2);
        auto publish = [&](auto phi) {
#pragma unroll
          for (int ft = 0; ft < FT; ++ft) {
            f4v bias[4];
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) bias[jj] = raw_to_f4<WT>(buf_load8(rB, (ROWS * wr + 32 * ft + 8 * jj + 4 * g) * 2));
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
#pragma unroll
              for (int t = 0; t < 2; ++t) {
                h8 r;
#pragma unroll
                for (int i = 0; i < 8; ++i) r[i] = (_Float16)phi(y[ft][tt][8 * t + i] + bias[2 * t + (i >> 2)][i & 3]);
                gtile[wt][FT * wr + ft][t][tt][lane] = r;
              }
          }
        };
        if (a.act == 0) publish([](float x) { return gelu_erf_f(x); });
        else if (a.act == 1) publish([](float x) { return gelu_tanh_f(x); });
        else publish([](float x) { return fmaxf(x, 0.f); });
      }
      commit_tile(parity ^ 1);
      __syncthreads();
      parity ^= 1;
    }
    // ================= phase B =================
    h8 gq[8][2];
#pragma unroll
    for (int fs = 0; fs < 8; ++fs)
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) gq[fs][tt] = gtile[wt][fs >> 1][fs & 1][tt][lane];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const bool lastB = s + 1 == NS;
      const bool more = !lastB || (c + 1 < nchunks);
      if (more) { if (!lastB) issue_tile(1, c, s + 1); else issue_tile(0, c + 1, 0); }
      const _Float16* wb = wt_lds[parity];
      if (s0 + s * kTile < s_end) {
#pragma unroll
        for (int fs = 0; fs < 8; ++fs) {
          h8 wf[FT];
#pragma unroll
          for (int rt = 0; rt < FT; ++rt) {
            const _Float16* q = wb + trB + 16 * fs * kTileRow + ROWS * wr + 32 * rt;
            wf[rt] = tr_frag(q, q + 8 * kTileRow);
          }
#pragma unroll
          for (int rt = 0; rt < FT; ++rt)
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) z[s][rt][tt] = mfma32(wf[rt], gq[fs][tt], z[s][rt][tt]);   // rows ranks, cols tokens
        }
      }
      if (more) commit_tile(parity ^ 1);
      __syncthreads();
      parity ^= 1;
    }
  }

  // ---- write Z fragment-major (fp16), 4 consecutive ranks per 8-byte store
  _Float16* Z = (_Float16*)a.Z;
#pragma unroll
  for (int tt = 0; tt < 2; ++tt) {
    const int tok = t0 + 64 * wt + 32 * tt + l32;
    if (tok >= T) continue;
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
      for (int rt = 0; rt < FT; ++rt)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const int r = s0 + s * kTile + ROWS * wr + 32 * rt + 8 * jj + 4 * g;
          if (r < s0 + slice_w && r < zch * 64) {   // ranks r2 .. 64*zch-1 are written as zeros (FM padding)
            const size_t unit = ((size_t)((tok >> 5) * zch + (r >> 6)) * 4 + ((r >> 3) & 3)) * 64 + ((r >> 5) & 1) * 32 + (tok & 31);
            h4 o;
#pragma unroll
            for (int i = 0; i < 4; ++i) o[i] = (_Float16)z[s][rt][tt][4 * jj + i];
            *(h4*)(Z + unit * 8 + 4 * ((r >> 2) & 1)) = o;
          }
        }
  }
}

template <int NS, int TG>
hipError_t launch_ns(const FfnCoreArgs& a, int nslices, int slice_w, hipStream_t s) {
  const dim3 grid(((a.T + 64 * TG - 1) / (64 * TG)) * nslices), block(256);
  if (a.w_dt == DT_F16) hipLaunchKernelGGL((ffn_core_kernel<NS, DT_F16, TG>), grid, block, 0, s, a, nslices, slice_w);
  else hipLaunchKernelGGL((ffn_core_kernel<NS, DT_BF16, TG>), grid, block, 0, s, a, nslices, slice_w);
  return hipGetLastError();
}

template <int TG>
hipError_t launch_tg(const FfnCoreArgs& a, int nslices, int slice_w, hipStream_t s) {
  switch ((slice_w + kTile - 1) / kTile) {
    case 1: return launch_ns<1, TG>(a, nslices, slice_w, s);
    case 2: return launch_ns<2, TG>(a, nslices, slice_w, s);
    case 3: return launch_ns<3, TG>(a, nslices, slice_w, s);
    case 4: return launch_ns<4, TG>(a, nslices, slice_w, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_ffn_core(const FfnCoreArgs& a, hipStream_t s) {
  const int nslices = (a.r2 + kMaxSlice - 1) / kMaxSlice;
  int slice_w = (a.r2 + nslices - 1) / nslices;
  slice_w = (slice_w + 63) / 64 * 64;
  // 128-token workgroups halve the weight traffic; 64-token ones fill the chip when tokens are few
  const long wg128 = (long)((a.T + 127) / 128) * nslices;
  return wg128 >= 224 ? launch_tg<2>(a, nslices, slice_w, s) : launch_tg<1>(a, nslices, slice_w, s);
}

}  // namespace fsvd
