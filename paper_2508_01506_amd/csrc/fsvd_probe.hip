// Measurement aid for the roofline: a loop of nothing but v_mfma_f32_32x32x16_f16 on register-resident operands, so that
// the benchmark can state the matrix-core rate this part sustains at the clock it holds under load next to the
// published peak.  Four independent accumulator chains per wavefront; nothing is read from memory.
#include "fsvd_common.h"
#include "fsvd_kernels.h"

namespace fsvd {

namespace {
__global__ void __launch_bounds__(256) mfma_probe_kernel(int iters, float* out) {
  const int lane = threadIdx.x & 63;
  h8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (_Float16)(0.001f * (float)((lane + i) & 15));
    b[i] = (_Float16)(0.002f * (float)((lane * 3 + i) & 7));
  }
  f16v c0 = zero16(), c1 = zero16(), c2 = zero16(), c3 = zero16();
  for (int it = 0; it < iters; ++it) {
    c0 = mfma32(a, b, c0);
    c1 = mfma32(a, b, c1);
    c2 = mfma32(a, b, c2);
    c3 = mfma32(a, b, c3);
  }
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = c0[0] + c1[5] + c2[10] + c3[15];   // keeps the chains alive
}
}  // namespace

hipError_t launch_mfma_probe(int workgroups, int iters, float* out, hipStream_t s) {
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(workgroups), dim3(256), 0, s, iters, out);
  return hipGetLastError();
}

}  // namespace fsvd
