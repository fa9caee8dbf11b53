// LayerNorm over the last axis (residual sums are formed in the producing GEMM's epilogue).
// One wavefront per token: the row lives in registers, mean and biased variance are two
// wavefront reductions in fp32, and the normalised row is written once (optionally in two
// formats: an fp32 copy for the residual stream and an fp16 copy that feeds the next MFMA).
// Memory-bound: one read and one or two writes of [T, D].
#include "fsvd_common.h"
#include "fsvd_kernels.h"

namespace fsvd {

constexpr int kLnMaxPerLane = 128;  // D <= 64 * 128

template <int PER_LANE>
__global__ void __launch_bounds__(256) layernorm_kernel(LayerNormArgs a) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= a.T) return;
  const int D = a.D;
  float x[PER_LANE];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < PER_LANE; ++i) {
    const int c = lane + 64 * i;
    x[i] = c < D ? load_param(a.X, (size_t)row * a.ldx + c, a.x_dt) : 0.f;
    sum += x[i];
  }
  const float mean = wave_sum(sum) / (float)D;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < PER_LANE; ++i) {
    const int c = lane + 64 * i;
    const float d = c < D ? x[i] - mean : 0.f;
    sq += d * d;
  }
  const float rstd = rsqrtf(wave_sum(sq) / (float)D + a.eps);
#pragma unroll
  for (int i = 0; i < PER_LANE; ++i) {
    const int c = lane + 64 * i;
    if (c < D) {
      const float y = (x[i] - mean) * rstd * load_param(a.gamma, c, a.p_dt) + load_param(a.beta, c, a.p_dt);
      store_out(a.Y0, (size_t)row * a.ldy0 + c, y, a.y0_dt);
      if (a.Y1) store_out(a.Y1, (size_t)row * a.ldy1 + c, y, a.y1_dt);
    }
  }
}

hipError_t launch_layernorm(const LayerNormArgs& a, hipStream_t s) {
  const dim3 grid((a.T + 3) / 4), block(256);
  const int per = (a.D + 63) / 64;
  if (per <= 4) hipLaunchKernelGGL(layernorm_kernel<4>, grid, block, 0, s, a);
  else if (per <= 16) hipLaunchKernelGGL(layernorm_kernel<16>, grid, block, 0, s, a);
  else if (per <= 32) hipLaunchKernelGGL(layernorm_kernel<32>, grid, block, 0, s, a);
  else if (per <= 64) hipLaunchKernelGGL(layernorm_kernel<64>, grid, block, 0, s, a);
  else if (per <= kLnMaxPerLane) hipLaunchKernelGGL(layernorm_kernel<kLnMaxPerLane>, grid, block, 0, s, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace fsvd
