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
// the tile's tokens; four buffers, requests three steps ahead.  The main loop has no compiler-tracked vector loads.
// Bias, gamma and beta of a wavefront's columns are staged as floats in LDS before the loop; the 32 x 32 patches of the
// epilogue reuse the weight ring.
#include "fsvd_common.h"
#include "fsvd_kernels.h"

namespace fsvd {

namespace {

// at most n of this wavefront's vector-memory operations outstanding (n a constant after unrolling; other values wait for all)
__device__ __forceinline__ void wait_vm(int n) {
  switch (n) {
    case 2: asm volatile("s_waitcnt vmcnt(2)" ::: "memory"); break;
    case 4: asm volatile("s_waitcnt vmcnt(4)" ::: "memory"); break;
    case 6: asm volatile("s_waitcnt vmcnt(6)" ::: "memory"); break;
    case 8: asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); break;
    case 12: asm volatile("s_waitcnt vmcnt(12)" ::: "memory"); break;
    default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
  }
}

template <int NT, int MT>   // NT = D / 256: 32-column tiles per wavefront; MT: 32-token tiles per workgroup
__global__ void __launch_bounds__(512, 1) linear_ln_kernel(LinearLnArgs a) {
  constexpr int NTD = 2 * NT;                       // 128-column tile images across D
  constexpr int NW = (4 * NTD) / 8;                 // weight requests per wavefront and step (4 NTD pieces of 1 KiB)
  constexpr int NB = 4;                             // ring of weight buffers: requests run 3 steps ahead of the MFMAs
  constexpr int kBufHalves = NTD * 16 * 128;        // one buffer: [column tile][16 rows x 128 columns]
  constexpr int NSLOT = NT < 2 ? 2 : NT;            // the epilogue reuses the ring: NSLOT blocks of 4 KiB per wavefront
  constexpr int kPatchHalves = 8 * NSLOT * 2048;
  static_assert(NSLOT * 4096 >= 32 * 36 * 4, "the padded fp32 patch fits a wavefront's share");
  __shared__ __attribute__((aligned(1024))) _Float16 wbuf[NB * kBufHalves > kPatchHalves ? NB * kBufHalves : kPatchHalves];
  __shared__ __attribute__((aligned(1024))) h8 abuf[NB][MT][64];               // [buffer][token tile][lane]: operand images
  __shared__ float red[8][32 * MT];
  __shared__ __attribute__((aligned(16))) float prm[8][3][32 * NT];            // per wavefront: bias, gamma, beta of its columns

  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int T = a.T, K = a.K, D = a.D;
  const int kch = (K + 63) / 64, nsteps = 4 * kch;
  const int tile0 = blockIdx.x * MT, ntiles = (T + 31) / 32;
  const int voff = lane * 16;
  const unsigned lds_w0 = lds_addr_of(&wbuf[0]), lds_a0 = lds_addr_of(&abuf[0][0][0]);
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
    if (wave < MT) lds_dma_wait_barrier<2 * (NW + 1)>();   // the next step's pieces are in; two steps' may be in flight
    else lds_dma_wait_barrier<2 * NW>();
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

  // the per-column parameters of this wavefront's columns, as floats, where the epilogue reads them with LDS latency
  const int colw = wave * 32 * NT;
  {
    float* const pw = &prm[wave][0][0];
#pragma unroll
    for (int c = lane; c < 32 * NT; c += 64) {
      pw[c] = a.bias ? load_param(a.bias, colw + c, a.w_dt) : 0.f;
      pw[32 * NT + c] = load_param(a.gamma, colw + c, a.p_dt);
      pw[64 * NT + c] = load_param(a.beta, colw + c, a.p_dt);
    }
  }

  request(0, 0);
  request(1, 1);
  request(2, 2);
  wait_barrier();
  int buf = 0;
  for (int s = 0; s < nsteps; ++s) {
    request((buf + NB - 1) & (NB - 1), s + NB - 1);
    const _Float16* wt = &wbuf[buf * kBufHalves];
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
    buf = (buf + 1) & (NB - 1);
  }
  lds_dma_wait_barrier<0>();                         // every wavefront's requests past the end have landed: LDS is quiet

  // ---- epilogue: + bias + residual, row statistics over all D columns, normalise, write.
  // The accumulators have lane = token; row-major tensors want lane = column (a wavefront then touches whole row
  // segments).  Both directions pass through this wavefront's share of the (now free) weight ring:
  //  - the residual's 32 x 32 blocks are requested straight into LDS, as they are stored (row-major, 64 or 128 bytes
  //    per row), up to NSLOT blocks ahead, and picked up per token from there;
  //  - the normalised block is written per token into a padded fp32 patch and read back along the rows.
  char* const ring = (char*)&wbuf[0] + wave * (NSLOT * 4096);
  const float* const pw = &prm[wave][0][0];
  const unsigned lds_ring = lds_addr_of(ring);
  const bool r32 = a.r_dt == DT_F32;
  const int res = r32 ? 4 : 2;                                // bytes per residual element
  const u4 rR = lds_dma_rsrc(uniform_ptr(a.R), a.R ? (unsigned)((size_t)T * D * res) : 0u);
  const int rrow = r32 ? lane >> 3 : lane >> 2;               // one request covers 8 (fp32) or 16 (16-bit) rows of a block
  const int rcol = r32 ? 16 * (lane & 7) : 16 * (lane & 3);   // this lane's 16 bytes inside the row's 128 or 64
  auto request_block = [&](int mt, int j, int slot) {         // rows past T: the last row again (never stored)
    const int tok0 = (tile0 + mt) * 32;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      if (d < res) {
        int tok = tok0 + rrow + (r32 ? 8 : 16) * d;
        tok = tok < T ? tok : T - 1;
        lds_dma16(rR, lds_ring + slot * 4096 + d * 1024, tok * D * res + rcol, (colw + 32 * j) * res);
      }
    }
  };
  constexpr int NBLK = MT * NT;
  if (a.R) {
#pragma unroll
    for (int i = 0; i < NSLOT && i < NBLK; ++i) request_block(i / NT, i % NT, i);
  }
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    float sum = 0.f;
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int i = mt * NT + j, slot = i % NSLOT;
      f4v rv[4];
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) rv[jj] = f4v{0.f, 0.f, 0.f, 0.f};
      if (a.R) {
        // requests complete in order: all but the blocks requested after this one have landed
        const int after = (i + NSLOT < NBLK ? i + NSLOT : NBLK) - 1 - i;
        if (r32) wait_vm(4 * after); else wait_vm(2 * after);
        const char* const sp = ring + slot * 4096;
        if (r32) {
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) rv[jj] = *(const f4v*)(sp + 128 * l32 + 32 * jj + 16 * g);
        } else {
          u2 raw[4];
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) raw[jj] = *(const u2*)(sp + 64 * l32 + 16 * jj + 8 * g);
#pragma unroll
          for (int jj = 0; jj < 4; ++jj)
            rv[jj] = a.r_dt == DT_BF16 ? raw_to_f4<DT_BF16>(raw[jj]) : raw_to_f4<DT_F16>(raw[jj]);
        }
        if (i + NSLOT < NBLK) {
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the slot has been read before it is requested into again
          request_block((i + NSLOT) / NT, (i + NSLOT) % NT, slot);
        }
      }
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const f4v b = *(const f4v*)(pw + 32 * j + 8 * jj + 4 * g);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          acc[mt][j][4 * jj + e] += b[e] + rv[jj][e];
          sum += acc[mt][j][4 * jj + e];
        }
      }
    }
    sum = halves_sum(sum);
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
    sq = halves_sum(sq);
    if (g == 0) red[wave][32 * mt + l32] = sq;
  }
  __syncthreads();

  // stores go through buffer resources: a lane whose token lies past T passes an out-of-range offset and writes nothing
  float* const po = (float*)ring;                             // [32 tokens][36]: 16-byte accesses from both sides
  const int prow = lane >> 3, pc4 = 4 * (lane & 7);           // row-major side: rows prow + 8 i, 4 columns from pc4
  const bool y32 = a.yrow_dt == DT_F32;
  const int yes = y32 ? 4 : 2;
  const rsrc_t rY = rsrc_at(a.Yrow, a.Yrow ? (long long)T * D * yes : 0, 0);
  const rsrc_t rF = rsrc_at(a.Yfm, a.Yfm ? (long long)fm_bytes(T, D) : 0, 0);
  const int cch = D / 64;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    float t = 0.f;
#pragma unroll
    for (int w2 = 0; w2 < 8; ++w2) t += red[w2][32 * mt + l32];
    const float rstd = rsqrtf(t / (float)D + a.eps);
    const int tok0 = (tile0 + mt) * 32;
    // fragment-major unit of (token, column n = colw + 32 j + 8 jj + 4 g): chunk n / 64, step jj, lane (n / 32) % 2 * 32 + token % 32
    const int fm_off = tok0 + l32 < T ? ((tile0 + mt) * cch * 256 + l32) * 16 + 8 * g : kOobOffset;
    int yoff[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int tk = tok0 + prow + 8 * i;
      yoff[i] = tk < T ? (tk * D + colw + pc4) * yes : kOobOffset;
    }
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int n0 = colw + 32 * j;
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const f4v gm = *(const f4v*)(pw + 32 * NT + 32 * j + 8 * jj + 4 * g);
        const f4v bt = *(const f4v*)(pw + 64 * NT + 32 * j + 8 * jj + 4 * g);
        f4v y;
#pragma unroll
        for (int e = 0; e < 4; ++e) y[e] = (acc[mt][j][4 * jj + e] - mean[mt]) * rstd * gm[e] + bt[e];
        if (a.Yfm) {
          h4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (_Float16)y[e];
          __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u2, o), rF, fm_off,
                                                (((n0 >> 6) * 4 + jj) * 64 + ((n0 >> 5) & 1) * 32) * 16, 0);
        }
        if (a.Yrow) *(f4v*)(po + l32 * 36 + 8 * jj + 4 * g) = y;
      }
      if (a.Yrow) {
        f4v yy[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) yy[i] = *(const f4v*)(po + (prow + 8 * i) * 36 + pc4);
        if (y32) {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u4, yy[i]), rY, yoff[i], 32 * j * 4, 0);
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            u2 raw;
            if (a.yrow_dt == DT_F16) {
              h4 h;
#pragma unroll
              for (int e = 0; e < 4; ++e) h[e] = (_Float16)yy[i][e];
              raw = __builtin_bit_cast(u2, h);
            } else {
              raw[0] = (uint32_t)float_to_bf16_bits(yy[i][0]) | ((uint32_t)float_to_bf16_bits(yy[i][1]) << 16);
              raw[1] = (uint32_t)float_to_bf16_bits(yy[i][2]) | ((uint32_t)float_to_bf16_bits(yy[i][3]) << 16);
            }
            __builtin_amdgcn_raw_buffer_store_b64(raw, rY, yoff[i], 32 * j * 2, 0);
          }
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

// the residual and the row-major output are addressed with 32-bit byte offsets below the out-of-range marker
bool linear_ln_fits(long long T, int D) { return T > 0 && T * D * 4 < (long long)kOobOffset; }

hipError_t launch_linear_ln(const LinearLnArgs& a, hipStream_t s) {
  if (!linear_ln_supported(a.D) || !linear_ln_fits(a.T, a.D)) return hipErrorInvalidValue;
  switch (a.D / 256) {
    case 1: return launch_nt<1>(a, s);
    case 2: return launch_nt<2>(a, s);
    case 3: return launch_nt<3>(a, s);
    default: return launch_nt<4>(a, s);
  }
}

}  // namespace fsvd
