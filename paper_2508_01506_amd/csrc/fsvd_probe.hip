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
// Delivery-rate probe: every workgroup streams `region_bytes` of `src` (the eight XCDs each get their own region, all
// workgroups of an XCD the same one, so after the first touch the data comes out of that XCD's L2) into LDS with the
// direct-to-LDS loads the fused kernels use: eight wavefronts, four 1 KiB loads each per step, two steps in flight,
// no barrier, optionally `reads` 16-byte LDS reads and `mfmas` MFMAs per wavefront and step as concurrent work.
template <int READS, int MFMAS>
__global__ void __launch_bounds__(512) dma_probe_kernel(const char* src, unsigned region_bytes, int steps, float* out) {
  constexpr int PER = 4, DEPTH = 2, STEP = 8 * PER * 1024;
  __shared__ __attribute__((aligned(1024))) unsigned char ring[DEPTH + 1][STEP];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const u4 r = lds_dma_rsrc(src + (size_t)(blockIdx.x & 7) * region_bytes, region_bytes);
  const unsigned lds0 = lds_addr_of(&ring[0][0]);
  unsigned soff = ((blockIdx.x >> 3) * 65536u) % region_bytes;      // region_bytes is a multiple of STEP
  soff -= soff % STEP;
  int slot = 0;
  auto request = [&]() {
#pragma unroll
    for (int p = 0; p < PER; ++p)
      lds_dma16(r, lds0 + slot * STEP + (wave * PER + p) * 1024, lane * 16, (int)(soff + (wave * PER + p) * 1024));
    soff += STEP;
    if (soff >= region_bytes) soff = 0;
    slot = slot == DEPTH ? 0 : slot + 1;
  };
  for (int d = 0; d < DEPTH; ++d) request();
  uint32_t acc = 0;
  h8 a8, b8;
#pragma unroll
  for (int i = 0; i < 8; ++i) { a8[i] = (_Float16)(float)(lane & 3); b8[i] = (_Float16)1.0f; }
  f16v c0 = zero16(), c1 = zero16();
  int rd = 0;
  for (int it = 0; it < steps; ++it) {
    request();
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(PER * DEPTH) : "memory");     // the step requested DEPTH steps ago has landed
    const u4* sl = (const u4*)ring[rd];
#pragma unroll
    for (int i = 0; i < READS; ++i) { const u4 v = sl[((wave * PER + (i % PER)) * 64 + lane)]; acc ^= v[0] ^ v[3]; }
#pragma unroll
    for (int m = 0; m < MFMAS / 2; ++m) { c0 = mfma32(a8, b8, c0); c1 = mfma32(a8, b8, c1); }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                        // the reads are done before the slot is requested again
    rd = rd == DEPTH ? 0 : rd + 1;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  out[(size_t)blockIdx.x * 512 + threadIdx.x] = (float)acc + c0[0] + c1[3];
}
}  // namespace

hipError_t launch_dma_probe(int workgroups, int steps, int with_work, const void* src, unsigned region_bytes, float* out, hipStream_t s) {
  if (with_work) hipLaunchKernelGGL((dma_probe_kernel<12, 8>), dim3(workgroups), dim3(512), 0, s, (const char*)src, region_bytes, steps, out);
  else hipLaunchKernelGGL((dma_probe_kernel<0, 0>), dim3(workgroups), dim3(512), 0, s, (const char*)src, region_bytes, steps, out);
  return hipGetLastError();
}

hipError_t launch_mfma_probe(int workgroups, int iters, float* out, hipStream_t s) {
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(workgroups), dim3(256), 0, s, iters, out);
  return hipGetLastError();
}

}  // namespace fsvd
