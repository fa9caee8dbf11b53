// Memory-bound helpers: LayerNorm over the last axis (the residual sums are formed in the
// producing GEMM's epilogue) and the row-major <-> fragment-major layout conversions.
//
// LayerNorm: one wavefront per token; each lane owns groups of 8 consecutive features (16- or
// 32-byte loads), the row stays in registers, mean and biased variance are two wavefront
// reductions in fp32.  The normalised row is written once row-major (any type; the fp32 residual
// stream) and/or once fragment-major in fp16 (the operand of the next MFMA), where a group of 8
// features is exactly one 16-byte unit.
#include "fsvd_common.h"
#include "fsvd_kernels.h"

namespace fsvd {

namespace {

// 8 consecutive elements starting at element index i (multiple of 8) of a typed array, as floats
__device__ __forceinline__ void load8(const void* p, size_t i, int dt, float (&x)[8]) {
  if (dt == DT_F32) {
    const f4v* q = (const f4v*)((const float*)p + i);
    const f4v lo = q[0], hi = q[1];
#pragma unroll
    for (int j = 0; j < 4; ++j) { x[j] = lo[j]; x[4 + j] = hi[j]; }
  } else {
    const u4 raw = *(const u4*)((const uint16_t*)p + i);
    if (dt == DT_F16) {
      const h8 h = __builtin_bit_cast(h8, raw);
#pragma unroll
      for (int j = 0; j < 8; ++j) x[j] = (float)h[j];
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) { x[2 * j] = __uint_as_float(raw[j] << 16); x[2 * j + 1] = __uint_as_float(raw[j] & 0xffff0000u); }
    }
  }
}
__device__ __forceinline__ void store8(void* p, size_t i, int dt, const float (&x)[8]) {
  if (dt == DT_F32) {
    f4v lo, hi;
#pragma unroll
    for (int j = 0; j < 4; ++j) { lo[j] = x[j]; hi[j] = x[4 + j]; }
    f4v* q = (f4v*)((float*)p + i);
    q[0] = lo; q[1] = hi;
  } else if (dt == DT_F16) {
    h8 h;
#pragma unroll
    for (int j = 0; j < 8; ++j) h[j] = (_Float16)x[j];
    *(h8*)((_Float16*)p + i) = h;
  } else {
    u4 raw;
#pragma unroll
    for (int j = 0; j < 4; ++j) raw[j] = (uint32_t)float_to_bf16_bits(x[2 * j]) | ((uint32_t)float_to_bf16_bits(x[2 * j + 1]) << 16);
    *(u4*)((uint16_t*)p + i) = raw;
  }
}
// element offset (in halves) of the 16-byte FM unit holding features k..k+7 (k multiple of 8) of token t
__device__ __forceinline__ size_t fm_unit_halves(int t, int k, int kchunks) {
  const int c = k >> 6, g = (k >> 5) & 1, kk = (k >> 3) & 3;
  return ((((size_t)(t >> 5) * kchunks + c) * 4 + kk) * 64 + g * 32 + (t & 31)) * 8;
}

template <int GROUPS>   // groups of 8 features per lane: D <= 512 * GROUPS
__global__ void __launch_bounds__(256) layernorm_kernel(LayerNormArgs a) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= a.T) return;
  const int D = a.D;
  float x[GROUPS][8];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < GROUPS; ++i) {
    const int k = 8 * (lane + 64 * i);
    if (k < D) {
      load8(a.X, (size_t)row * D + k, a.x_dt, x[i]);
#pragma unroll
      for (int j = 0; j < 8; ++j) sum += x[i][j];
    }
  }
  const float mean = wave_sum(sum) / (float)D;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < GROUPS; ++i)
    if (8 * (lane + 64 * i) < D) {
#pragma unroll
      for (int j = 0; j < 8; ++j) { const float d = x[i][j] - mean; sq += d * d; }
    }
  const float rstd = rsqrtf(wave_sum(sq) / (float)D + a.eps);
  const int kchunks = (D + 63) / 64;
#pragma unroll
  for (int i = 0; i < GROUPS; ++i) {
    const int k = 8 * (lane + 64 * i);
    if (k < D) {
      float gm[8], bt[8], y[8];
      load8(a.gamma, k, a.p_dt, gm);
      load8(a.beta, k, a.p_dt, bt);
#pragma unroll
      for (int j = 0; j < 8; ++j) y[j] = (x[i][j] - mean) * rstd * gm[j] + bt[j];
      if (a.Yrow) store8(a.Yrow, (size_t)row * D + k, a.yrow_dt, y);
      if (a.Yfm) store8(a.Yfm, fm_unit_halves(row, k, kchunks), DT_F16, y);
    }
  }
}

// one thread per 16-byte FM unit
__global__ void __launch_bounds__(256) pack_fm_kernel(const void* src, int src_dt, int T, int K, _Float16* dst, size_t units) {
  const size_t u = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (u >= units) return;
  const int kchunks = (K + 63) / 64;
  const int lane = u & 63, kk = (u >> 6) & 3;
  const size_t blk = u >> 8;
  const int c = blk % kchunks, tile = blk / kchunks;
  const int t = tile * 32 + (lane & 31), k = 64 * c + 32 * (lane >> 5) + 8 * kk;
  if (src_dt == DT_BF16) {   // the widening every kernel applies to bf16 operands (toward zero: saturates, never infinite)
    u4 raw = {0u, 0u, 0u, 0u};
    if (t < T && k < K) raw = *(const u4*)((const uint16_t*)src + (size_t)t * K + k);
    *(h8*)(dst + u * 8) = raw_to_h8<DT_BF16>(raw);
    return;
  }
  float x[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (t < T && k < K) load8(src, (size_t)t * K + k, src_dt, x);
  store8(dst, u * 8, DT_F16, x);
}
// one thread per 16 bytes of the tile images: destination unit d of a tile is row d / 16, stored segment (d / 4) % 4
__global__ void __launch_bounds__(256) pack_tiled_kernel(const void* src, int src_dt, int K, int N, _Float16* dst, size_t units) {
  const size_t u = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (u >= units) return;
  const int ntn = (N + 127) / 128;
  const size_t tile = u >> 11;
  const int d = (int)(u & 2047);
  const int row = d >> 4, seg = ((d >> 2) & 3) ^ (row & 3);
  const int k = (int)(tile / ntn) * 128 + row, n = (int)(tile % ntn) * 128 + 32 * seg + 8 * (d & 3);
  u4 raw = {0u, 0u, 0u, 0u};
  if (k < K && n < N) raw = *(const u4*)((const uint16_t*)src + (size_t)k * N + n);
  // the conversion the kernels apply when they stage row-major weights, so both layouts give the same bits
  *(h8*)(dst + u * 8) = src_dt == DT_BF16 ? raw_to_h8<DT_BF16>(raw) : raw_to_h8<DT_F16>(raw);
}
__global__ void __launch_bounds__(256) unpack_fm_kernel(const _Float16* src, int T, int K, void* dst, int dst_dt, size_t groups) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;   // group of 8 features
  if (i >= groups) return;
  const int kg = K / 8;
  const int t = i / kg, k = 8 * (i % kg);
  float x[8];
  load8(src, fm_unit_halves(t, k, (K + 63) / 64), DT_F16, x);
  store8(dst, (size_t)t * K + k, dst_dt, x);
}

}  // namespace

hipError_t launch_layernorm(const LayerNormArgs& a, hipStream_t s) {
  const dim3 grid((a.T + 3) / 4), block(256);
  const int groups = (a.D + 511) / 512;
  if (groups <= 1) hipLaunchKernelGGL(layernorm_kernel<1>, grid, block, 0, s, a);
  else if (groups <= 2) hipLaunchKernelGGL(layernorm_kernel<2>, grid, block, 0, s, a);
  else if (groups <= 4) hipLaunchKernelGGL(layernorm_kernel<4>, grid, block, 0, s, a);
  else if (groups <= 8) hipLaunchKernelGGL(layernorm_kernel<8>, grid, block, 0, s, a);
  else if (groups <= 16) hipLaunchKernelGGL(layernorm_kernel<16>, grid, block, 0, s, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_pack_fm(const void* src, int src_dt, int T, int K, void* dst_fm, hipStream_t s) {
  const size_t units = fm_bytes(T, K) / 16;
  hipLaunchKernelGGL(pack_fm_kernel, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, s, src, src_dt, T, K,
                     (_Float16*)dst_fm, units);
  return hipGetLastError();
}
hipError_t launch_pack_tiled(const void* src, int src_dt, int K, int N, void* dst, hipStream_t s) {
  const size_t units = tiled_bytes(K, N) / 16;
  hipLaunchKernelGGL(pack_tiled_kernel, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, s, src, src_dt, K, N,
                     (_Float16*)dst, units);
  return hipGetLastError();
}
hipError_t launch_unpack_fm(const void* src_fm, int T, int K, void* dst, int dst_dt, hipStream_t s) {
  const size_t groups = (size_t)T * (K / 8);
  hipLaunchKernelGGL(unpack_fm_kernel, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, s, (const _Float16*)src_fm, T, K,
                     dst, dst_dt, groups);
  return hipGetLastError();
}

}  // namespace fsvd
