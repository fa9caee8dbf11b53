// Up-projection fused with the residual add and the LayerNorm that follows it (the H3 -> H4 and H7 -> H8 hand-offs of
// a post-LN layer):   Y = LN(A W + bias + R),  A [T, K] fragment-major fp16 (rank space), W [K, D] prepacked tile images.
// The paper only notes that the residual add and the normalisation remain once the two blocks are fused; done as
// separate passes they cost a write and a read of the [T, D] fp32 stream each, more than the projection itself when
// the rank is small.  Here one workgroup owns 32 MT tokens and ALL D columns (D <= 1024, D % 256 == 0), so the row
// statistics are available on chip: wavefront w accumulates columns [w D / 8, (w + 1) D / 8) for all tokens
// (accumulators: lane = token, registers = columns, as in linear_kernel), per-lane partial sums are combined through LDS,
// and the normalised row is written once - fp32 / 16-bit row-major and / or the fragment-major fp16 copy that feeds the
// next projection.
// Operands reach LDS by direct loads (see fsvd_common.h): per step of 16 contraction rows, 16 rows x D columns of the
// weight tile images (the two 8-row groups an MFMA step of the fragment-major slot order touches) and the A operands of
// the tile's tokens; three buffers, requests two steps ahead.  The main loop has no compiler-tracked vector loads.
#include "fsvd_common.h"
#include "fsvd_kernels.h"

namespace fsvd {

namespace {

template <int NT, int MT>   // NT = D / 256: 32-column tiles per wavefront; MT: 32-token tiles per workgroup
__global__ void __launch_bounds__(512, 1) linear_ln_kernel(LinearLnArgs a) {
  constexpr int NTD = 2 * NT;                       // 128-column tile images across D
  constexpr int NW = (4 * NTD) / 8;                 // weight requests per wavefront and step (4 NTD pieces of 1 KiB)
  __shared__ __attribute__((aligned(1024))) _Float16 wbuf[3][NTD][16 * 128];   // [buffer][column tile][16 rows x 128 columns]
  __shared__ __attribute__((aligned(1024))) h8 abuf[3][MT][64];                // [buffer][token tile][lane]: operand images
  __shared__ float red[8][32 * MT];
  __shared__ float patch[8][32 * 33];              // per wavefront: one 32 x 32 block in transit between the two lane orders

  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int T = a.T, K = a.K, D = a.D;
  const int kch = (K + 63) / 64, nsteps = 4 * kch;
  const int tile0 = blockIdx.x * MT, ntiles = (T + 31) / 32;
  const int voff = lane * 16;
  const unsigned lds_w0 = lds_addr_of(&wbuf[0][0][0]), lds_a0 = lds_addr_of(&abuf[0][0][0]);
  const u4 rW = lds_dma_rsrc(uniform_ptr(a.W), (unsigned)tiled_bytes(K, D));
  const u4 rA = lds_dma_rsrc(uniform_ptr(a.A), (unsigned)fm_bytes(T, K));

  // step s = (chunk c = s / 4, MFMA step kk = s % 4): contraction rows 64 c + 8 kk + {0..7} and 64 c + 32 + 8 kk + {0..7}
  auto request = [&](int buf, int s) {
    s = s < nsteps ? s : nsteps - 1;                // past the end: the last step again (never consumed)
    const int c = s >> 2, kk = s & 3;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
      const int q = wave + 8 * i;                   // piece: column tile q / 4, row group (q / 2) % 2, 4-row part q % 2
      const int nt = q >> 2, h = (q >> 1) & 1, part = q & 1;
      const int row = 64 * (c & 1) + 32 * h + 8 * kk + 4 * part;      // first of 4 rows inside the 128-row tile image
      lds_dma16(rW, lds_w0 + ((buf * NTD + nt) * 16 + 8 * h + 4 * part) * 256, voff,
                ((c >> 1) * NTD + nt) * kTileImageBytes + row * 256);
    }
    if (wave < MT) {
      int tile = tile0 + wave;
      tile = tile < ntiles ? tile : ntiles - 1;     // token tiles past the end: any valid one (their rows are not stored)
      lds_dma16(rA, lds_a0 + (buf * MT + wave) * 1024, voff, ((tile * kch + c) * 4 + kk) * 1024);
    }
  };
  auto wait_barrier = [&]() {
    if (wave < MT) lds_dma_wait_barrier<NW + 1>();
    else lds_dma_wait_barrier<NW>();
  };

  f16v acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[mt][j] = zero16();

  // this wavefront's columns: 32 NT columns from wave * 32 NT; tile j sits in column tile image (col / 128), segment (col % 128) / 32
  int troff[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int col = wave * 32 * NT + 32 * j;
    troff[j] = (col >> 7) * (16 * 128) + tr_lane_off_swz(lane, (col & 127) >> 5) + 8 * g * 128;
  }

  request(0, 0);
  request(1, 1);
  wait_barrier();
  int buf = 0;
  for (int s = 0; s < nsteps; ++s) {
    const int b2 = buf >= 1 ? buf - 1 : 2;          // (buf + 2) % 3
    request(b2, s + 2);
    const _Float16* wt = &wbuf[buf][0][0];
    h8 bf[NT], af[MT];
#pragma unroll
    for (int j = 0; j < NT; ++j) bf[j] = tr_frag(wt + troff[j], wt + troff[j] + 4 * 128);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) af[mt] = abuf[buf][mt][lane];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int j = 0; j < NT; ++j) acc[mt][j] = mfma32(bf[j], af[mt], acc[mt][j]);   // rows columns, cols tokens
    wait_barrier();
    buf = buf == 2 ? 0 : buf + 1;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the requests past the end have landed: LDS is quiet

  // ---- epilogue: + bias + residual, row statistics over all D columns, normalise, write.
  // The accumulators have lane = token; row-major tensors want lane = column (a wavefront then touches 128-byte row
  // segments).  Each 32 x 32 block therefore passes through a wavefront-private LDS patch: the residual is read from
  // memory 16 bytes per lane along the rows and picked up per token, the result goes the other way.
  float* const pt = &patch[wave][0];
  const int prow = lane >> 3, pc4 = 4 * (lane & 7);          // row-major side: rows prow + 8 i, 4 columns from pc4
  const int colw = wave * 32 * NT;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int tok0 = (tile0 + mt) * 32;
    float sum = 0.f;
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      if (a.R) {
        f4v rr[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int tok = tok0 + prow + 8 * i;
          rr[i] = tok < T ? load4(a.R, (size_t)tok * D + colw + 32 * j + pc4, a.r_dt) : f4v{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int e = 0; e < 4; ++e) pt[(prow + 8 * i) * 33 + pc4 + e] = rr[i][e];
      }
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const int n = colw + 32 * j + 8 * jj + 4 * g;
        const f4v b = a.bias ? load4(a.bias, n, a.w_dt) : f4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float r = a.R ? pt[l32 * 33 + 8 * jj + 4 * g + e] : 0.f;
          acc[mt][j][4 * jj + e] += b[e] + r;
          sum += acc[mt][j][4 * jj + e];
        }
      }
    }
    sum += __shfl_xor(sum, 32, 64);
    if (g == 0) red[wave][32 * mt + l32] = sum;
  }
  __syncthreads();
  float mean[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    float t = 0.f;
#pragma unroll
    for (int w2 = 0; w2 < 8; ++w2) t += red[w2][32 * mt + l32];
    mean[mt] = t / (float)D;
  }
  __syncthreads();
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    float sq = 0.f;
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float dlt = acc[mt][j][v] - mean[mt];
        sq = fmaf(dlt, dlt, sq);
      }
    sq += __shfl_xor(sq, 32, 64);
    if (g == 0) red[wave][32 * mt + l32] = sq;
  }
  __syncthreads();
  const int cch = D / 64;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    float t = 0.f;
#pragma unroll
    for (int w2 = 0; w2 < 8; ++w2) t += red[w2][32 * mt + l32];
    const float rstd = rsqrtf(t / (float)D + a.eps);
    const int tok0 = (tile0 + mt) * 32, tok = tok0 + l32;
#pragma unroll
    for (int j = 0; j < NT; ++j) {
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const int n = colw + 32 * j + 8 * jj + 4 * g;
        const f4v gm = load4(a.gamma, n, a.p_dt), bt = load4(a.beta, n, a.p_dt);
        f4v y;
#pragma unroll
        for (int e = 0; e < 4; ++e) y[e] = (acc[mt][j][4 * jj + e] - mean[mt]) * rstd * gm[e] + bt[e];
        if (a.Yfm && tok < T) {
          const size_t unit = ((size_t)((tok >> 5) * cch + (n >> 6)) * 4 + ((n >> 3) & 3)) * 64 + ((n >> 5) & 1) * 32 + (tok & 31);
          h4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (_Float16)y[e];
          *(h4*)((_Float16*)a.Yfm + unit * 8 + 4 * ((n >> 2) & 1)) = o;
        }
        if (a.Yrow) {
#pragma unroll
          for (int e = 0; e < 4; ++e) pt[l32 * 33 + 8 * jj + 4 * g + e] = y[e];
        }
      }
      if (a.Yrow) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int tk = tok0 + prow + 8 * i;
          f4v y;
#pragma unroll
          for (int e = 0; e < 4; ++e) y[e] = pt[(prow + 8 * i) * 33 + pc4 + e];
          if (tk < T) store4(a.Yrow, (size_t)tk * D + colw + 32 * j + pc4, y, a.yrow_dt);
        }
      }
    }
  }
}

template <int NT>
hipError_t launch_nt(const LinearLnArgs& a, hipStream_t s) {
  // 64-token workgroups when that still gives one per compute unit, else 32-token ones
  if ((a.T + 63) / 64 >= 256) hipLaunchKernelGGL((linear_ln_kernel<NT, 2>), dim3((a.T + 63) / 64), dim3(512), 0, s, a);
  else hipLaunchKernelGGL((linear_ln_kernel<NT, 1>), dim3((a.T + 31) / 32), dim3(512), 0, s, a);
  return hipGetLastError();
}

}  // namespace

bool linear_ln_supported(int D) { return D % 256 == 0 && D >= 256 && D <= 1024; }

hipError_t launch_linear_ln(const LinearLnArgs& a, hipStream_t s) {
  if (!linear_ln_supported(a.D)) return hipErrorInvalidValue;
  switch (a.D / 256) {
    case 1: return launch_nt<1>(a, s);
    case 2: return launch_nt<2>(a, s);
    case 3: return launch_nt<3>(a, s);
    default: return launch_nt<4>(a, s);
  }
}

}  // namespace fsvd
