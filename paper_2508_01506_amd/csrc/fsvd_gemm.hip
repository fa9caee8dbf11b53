// C[T, N] = A[T, K] W[K, N] (+ bias) (+ residual): the rank projections P_a = X U_a, the factored
// output projection (C U_o) V_o + b_o and the two GEMMs that bracket the fused FFN kernel
// (Alg. 2 "GEMM 1st" / "GEMM 2nd").
//
// One workgroup = 4 wavefronts stacked along the rows: a 256 x BN output tile, each wavefront a
// 64 x BN slab held as 32x32 MFMA accumulators.  Activation fragments are loaded straight from
// global memory into registers (every lane reads 64 contiguous bytes of its own row per 64-wide
// contraction chunk; no other wavefront needs them), weight tiles are transposed in registers and
// double-buffered in LDS, where all four wavefronts read them.  LDS read traffic is 0.5 KiB per MFMA.
#include "fsvd_common.h"
#include "fsvd_kernels.h"

namespace fsvd {

template <int AT> struct RawAct { u4 v; };
template <> struct RawAct<DT_F32> { f4v lo, hi; };

template <int AT>
__device__ __forceinline__ RawAct<AT> load_raw_act(const void* row, int k, bool ok) {
  RawAct<AT> r;
  if constexpr (AT == DT_F32) {
    f4v z = {0.f, 0.f, 0.f, 0.f};
    r.lo = z; r.hi = z;
    if (ok) { const f4v* p = (const f4v*)((const float*)row + k); r.lo = p[0]; r.hi = p[1]; }
  } else {
    u4 z = {0u, 0u, 0u, 0u};
    r.v = z;
    if (ok) r.v = *(const u4*)((const uint16_t*)row + k);
  }
  return r;
}
template <int AT>
__device__ __forceinline__ h8 cvt_raw_act(const RawAct<AT>& r) {
  if constexpr (AT == DT_F32) {
    h8 o;
    o[0] = (_Float16)r.lo[0]; o[1] = (_Float16)r.lo[1]; o[2] = (_Float16)r.lo[2]; o[3] = (_Float16)r.lo[3];
    o[4] = (_Float16)r.hi[0]; o[5] = (_Float16)r.hi[1]; o[6] = (_Float16)r.hi[2]; o[7] = (_Float16)r.hi[3];
    return o;
  } else {
    return raw_to_h8<AT>(r.v);
  }
}

template <int AT, int WT, int BN>
__global__ void __launch_bounds__(256, (AT == DT_F32 && BN == 128) ? 1 : 2) linear_kernel(LinearArgs a, int tiles_m, int tiles_n) {
  constexpr int NT = BN / 32;                       // 32-column MFMA tiles per wavefront
  constexpr int STAGE_WAVES = BN / 32;              // wavefronts that stage the weight tile
  __shared__ __attribute__((aligned(16))) _Float16 lds[2][BN * kLdsRow];

  const int tile = xcd_tile(blockIdx.x, tiles_m * tiles_n);
  const int tm = tile / tiles_n;
  int tn = tile % tiles_n;
  int gi = 0;
  for (; gi < a.ngroups - 1; ++gi) {
    int t = (a.g[gi].N + BN - 1) / BN;
    if (tn < t) break;
    tn -= t;
  }
  const LinearGroup G = a.g[gi];
  const int n0 = tn * BN;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int m0 = tm * 256 + wave * 64;
  const int K = a.K;

  // activation row pointers (rows beyond T are clamped; their results are never stored)
  const char* arow[2];
  const size_t esz = (AT == DT_F32) ? 4 : 2;
#pragma unroll
  for (int mt = 0; mt < 2; ++mt) {
    int r = m0 + 32 * mt + l32;
    r = r < a.T ? r : a.T - 1;
    arow[mt] = (const char*)a.A + (size_t)r * a.lda * esz;
  }
  // weight staging coordinates
  const int s_ng = (lane & 3) + 4 * wave;   // 8-column group inside the tile
  const int s_q = lane >> 2;                // 4-row group inside the chunk
  const bool stager = wave < STAGE_WAVES;

  f16v acc[2][NT];
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = zero16();

  RawAct<AT> a_raw[2][4];
  h8 a_frag[2][4];
  u4 w_raw[4];

  const int nchunks = (K + kChunkK - 1) / kChunkK;

  auto load_a = [&](int c) {
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        int k = c * kChunkK + chunk_off(kk, g);
        a_raw[mt][kk] = load_raw_act<AT>(arow[mt], k, k < K);
      }
  };
  auto cvt_a = [&]() {
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) a_frag[mt][kk] = cvt_raw_act<AT>(a_raw[mt][kk]);
  };
  auto load_w = [&](int c) {
    if (stager) load_w4x8<WT>(G.W, (size_t)G.ldw, c * kChunkK + 4 * s_q, n0 + 8 * s_ng, K, G.N, w_raw);
  };
  auto store_w = [&](int buf) {
    if (stager) {
      u2 t[8];
      transpose_w4x8<WT>(w_raw, t);
#pragma unroll
      for (int j = 0; j < 8; ++j) *(u2*)&lds[buf][(8 * s_ng + j) * kLdsRow + 4 * s_q] = t[j];
    }
  };

  load_a(0);
  load_w(0);
  cvt_a();
  store_w(0);
  __syncthreads();

  for (int c = 0; c < nchunks; ++c) {
    const bool more = c + 1 < nchunks;
    if (more) { load_a(c + 1); load_w(c + 1); }
    const _Float16* wt = lds[c & 1];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      h8 bf[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) bf[nt] = *(const h8*)&wt[(32 * nt + l32) * kLdsRow + chunk_off(kk, g)];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = mfma32(a_frag[mt][kk], bf[nt], acc[mt][nt]);
    }
    if (more) { store_w((c + 1) & 1); cvt_a(); }
    __syncthreads();
  }

  // epilogue
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int col = n0 + 32 * nt + l32;
    if (col >= G.N) continue;
    const float bias = G.bias ? load_param(G.bias, col, a.w_dt) : 0.f;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + 32 * mt + 8 * (v >> 2) + 4 * g + (v & 3);
        if (row < a.T) {
          float x = acc[mt][nt][v] + bias;
          if (a.R) x += load_param(a.R, (size_t)row * a.ldr + col, a.r_dt);
          store_out(G.C, (size_t)row * G.ldc + col, x, a.c_dt);
        }
      }
  }
}

template <int AT, int WT>
static hipError_t launch_bn(const LinearArgs& a, hipStream_t s) {
  const int tiles_m = (a.T + 255) / 256;
  int n128 = 0, n64 = 0;
  for (int i = 0; i < a.ngroups; ++i) { n128 += (a.g[i].N + 127) / 128; n64 += (a.g[i].N + 63) / 64; }
  // narrow tiles when the wide ones would leave compute units idle
  const bool narrow = (long)tiles_m * n128 < 320;
  if (narrow) {
    hipLaunchKernelGGL((linear_kernel<AT, WT, 64>), dim3(tiles_m * n64), dim3(256), 0, s, a, tiles_m, n64);
  } else {
    hipLaunchKernelGGL((linear_kernel<AT, WT, 128>), dim3(tiles_m * n128), dim3(256), 0, s, a, tiles_m, n128);
  }
  return hipGetLastError();
}

hipError_t launch_linear(const LinearArgs& a, hipStream_t s) {
  if (a.w_dt == DT_F16) {
    if (a.a_dt == DT_F16) return launch_bn<DT_F16, DT_F16>(a, s);
    if (a.a_dt == DT_F32) return launch_bn<DT_F32, DT_F16>(a, s);
    return launch_bn<DT_BF16, DT_F16>(a, s);
  } else {
    if (a.a_dt == DT_F16) return launch_bn<DT_F16, DT_BF16>(a, s);
    if (a.a_dt == DT_F32) return launch_bn<DT_F32, DT_BF16>(a, s);
    return launch_bn<DT_BF16, DT_BF16>(a, s);
  }
}

}  // namespace fsvd
