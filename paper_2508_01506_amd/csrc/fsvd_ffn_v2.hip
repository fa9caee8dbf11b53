// FlashSVDFFN V2 (Alg. 3): the whole factored FFN of a block of tokens in one kernel,
//   out = phi((X U_1) V_1 + b_1) U_2 V_2 + b_2,
// with the rank projection X U_1 and the up-projection Z V_2 done inside the kernel as well, so that neither the
// rank-space activations P1 = X U_1 and Z nor the hidden activation ever exist in device memory: the kernel reads X and
// the four factor matrices and writes the result, and needs no workspace.
//
// One workgroup (8 wavefronts) owns 32 MT tokens and runs a chain of four products of the same shape,
//   Out^T [N, tokens] = W^T [N, K] . In^T [K, tokens],
// "transposed" so that tokens lie along the lanes: the accumulators of one product, rounded to fp16, are the operand
// registers of the next.  The activations between two products stay in LDS as ready operand fragments
// ([16-wide contraction step][token tile][lane] x 16 bytes): X is staged in slabs of 512 / MT columns, P1^T (later Z^T) takes
// 64 KiB, the activated hidden chunk (512 / MT features) 32 KiB.  All weights are prepacked tile images; one step of
// 16 contraction rows x 512 columns (16 KiB) at a time is copied straight into LDS, three buffers, two steps ahead, as
// ONE request stream over the whole kernel (a cursor walks the same loop nest as the consumers), so that the copies never
// drain between the products.  Within a 512-column slab wavefront w owns columns 64 w .. 64 w + 63.
//   step 1: P1^T = U_1^T X^T                         (sum over D in slabs; all slabs of r1 per X slab)
//   step 2: per chunk of F: H^T = V_1^T P1^T + b_1, G = phi(H) -> LDS;  Z^T += U_2^T G^T  (Z^T stays in registers)
//   step 3: out^T = V_2^T Z^T + b_2 per 512-column slab of D, written row-major.
// Limits: r1, r2 <= 1024 / MT (the register and LDS budget of Z^T and P1^T).
#include "fsvd_common.h"
#include "fsvd_kernels.h"

namespace fsvd {

namespace {

constexpr int kV2Threads = 512;
constexpr int kV2StepBytes = 16 * 512 * 2;     // one staged step: 4 tile images x 16 rows x 256 bytes

// The request stream of the kernel below: which 16-row x 512-column step of which factor matrix is copied into LDS
// next.  The cursor walks the loop nest of the four products in the order in which the consumer loops use the steps;
// all of it is wave-uniform (scalar registers).
template <int MT>
struct WeightStream {
  static constexpr int KS = 32 / MT, FC = 16 * KS;
  u4 rs_u1, rs_v1, rs_u2, rs_v2;               // buffer descriptors of the four tile-image arrays
  int ntn_u1, ntn_v1, ntn_u2, ntn_v2;          // tile images per row of tiles
  int D, F, nxs, nsl1, nk1, nch, nsl2, nk2, nds;
  int ph, i0, i1, ks;                          // cursor: product, outer index (X slab, chunk of F, slab of D), rank slab, step
  int buf;                                     // buffer of the step being consumed
  int wave, voff;
  unsigned lds_w0;

  __device__ __forceinline__ int steps_in(int total, int part) const {   // 16-row steps of part `part` (FC wide) of an axis
    const int k = (total - FC * part + 15) / 16;
    return k < KS ? k : KS;
  }
  __device__ __forceinline__ void init(const FfnV2Args& a, int wave_, int lane, unsigned lds_w0_) {
    D = a.D; F = a.F;
    rs_u1 = lds_dma_rsrc(a.U1, (unsigned)tiled_bytes(a.D, a.r1));
    rs_v1 = lds_dma_rsrc(a.V1, (unsigned)tiled_bytes(a.r1, a.F));
    rs_u2 = lds_dma_rsrc(a.U2, (unsigned)tiled_bytes(a.F, a.r2));
    rs_v2 = lds_dma_rsrc(a.V2, (unsigned)tiled_bytes(a.r2, a.D));
    ntn_u1 = (a.r1 + 127) / 128; ntn_v1 = (a.F + 127) / 128; ntn_u2 = (a.r2 + 127) / 128; ntn_v2 = (a.D + 127) / 128;
    nxs = (a.D + FC - 1) / FC; nsl1 = (a.r1 + 511) / 512; nk1 = (a.r1 + 15) / 16;
    nch = (a.F + FC - 1) / FC; nsl2 = (a.r2 + 511) / 512; nk2 = (a.r2 + 15) / 16;
    nds = (a.D + 511) / 512;
    ph = i0 = i1 = ks = 0; buf = 0;
    wave = wave_; voff = lane * 16; lds_w0 = lds_w0_;
  }
  __device__ __forceinline__ void request(int b) const {
    u4 rs; int ntn, k, n0, nimg = 4;
    if (ph == 0)      { rs = rs_u1; ntn = ntn_u1; k = FC * i0 + 16 * ks; n0 = 512 * i1; }
    else if (ph == 1) { rs = rs_v1; ntn = ntn_v1; k = 16 * ks; n0 = FC * i0; nimg = FC / 128; }
    else if (ph == 2) { rs = rs_u2; ntn = ntn_u2; k = FC * i0 + 16 * ks; n0 = 512 * i1; }
    else if (ph == 3) { rs = rs_v2; ntn = ntn_v2; k = 16 * ks; n0 = 512 * i0; }
    else              { rs = rs_v2; ntn = ntn_v2; k = 0; n0 = 0; }            // past the end: never consumed
#pragma unroll
    for (int i = 0; i < 4; ++i) rs[i] = __builtin_amdgcn_readfirstlane(rs[i]);   // the selected descriptor stays in scalar registers
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int q = (wave + 8 * i) & (4 * nimg - 1);   // piece: tile image q / 4, 4-row part q % 4 (narrow steps: twice the same)
      int nt = (n0 >> 7) + (q >> 2);
      nt = nt < ntn ? nt : ntn - 1;                    // images right of the matrix: any valid one (their columns are not used)
      lds_dma16(rs, lds_w0 + b * kV2StepBytes + (q >> 2) * 4096 + (q & 3) * 1024, voff,
                ((k >> 7) * ntn + nt) * kTileImageBytes + ((k & 127) + 4 * (q & 3)) * 256);
    }
  }
  __device__ __forceinline__ void advance() {
    ++ks;
    if (ph == 0) {
      if (ks == steps_in(D, i0)) { ks = 0; if (++i1 == nsl1) { i1 = 0; if (++i0 == nxs) { i0 = 0; ph = 1; } } }
    } else if (ph == 1) {
      if (ks == nk1) { ks = 0; i1 = 0; ph = 2; }
    } else if (ph == 2) {
      if (ks == steps_in(F, i0)) {
        ks = 0;
        if (++i1 == nsl2) { i1 = 0; if (++i0 == nch) { i0 = 0; ph = 3; } else ph = 1; }
      }
    } else if (ph == 3) {
      if (ks == nk2) { ks = 0; if (++i0 == nds) ph = 4; }
    }
    ph = __builtin_amdgcn_readfirstlane(ph); i0 = __builtin_amdgcn_readfirstlane(i0);
    i1 = __builtin_amdgcn_readfirstlane(i1); ks = __builtin_amdgcn_readfirstlane(ks);
  }
  __device__ __forceinline__ void start() {      // the first two steps; returns with step 0 in LDS
    request(0); advance();
    request(1); advance();
    lds_dma_wait_barrier<2>();
  }
  __device__ __forceinline__ void begin_step() {
    request(buf >= 1 ? buf - 1 : 2);             // (buf + 2) % 3: read during the step before this one, free since its barrier
    advance();
  }
  __device__ __forceinline__ void end_step() {
    lds_dma_wait_barrier<2>();                   // all but the newest request have landed: the next step's rows are in LDS
    buf = buf == 2 ? 0 : buf + 1;
  }
};

template <int MT>
__global__ void __launch_bounds__(kV2Threads, 1) ffn_v2_kernel(FfnV2Args a) {
  constexpr int KS = 32 / MT;                  // contraction steps per X slab and per chunk of F (gfr holds KS * MT fragments)
  constexpr int FC = 16 * KS;                  // chunk of F, and X slab width
  constexpr int NTA = 2 / MT;                  // 32-feature tiles per wavefront in the hidden product
  constexpr int NSL = 2 / MT;                  // 512-column slabs of the ranks
  __shared__ __attribute__((aligned(16))) h8 pfr[64][64];                  // P1^T, later Z^T: [step * MT + tile][lane]
  __shared__ __attribute__((aligned(16))) h8 gfr[32][64];                  // X slab, later the activated chunk
  __shared__ __attribute__((aligned(16))) _Float16 wbuf[3][4][16][128];    // [buffer][tile image][row][column]

  const int tid = threadIdx.x;
  const int lane = tid & 63, l32 = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int T = a.T, D = a.D, F = a.F, r1 = a.r1, r2 = a.r2;
  const int tok0 = blockIdx.x * 32 * MT;

  WeightStream<MT> ws;
  ws.init(a, wave, lane, lds_addr_of(&wbuf[0][0][0][0]));
  const int nxs = ws.nxs, nsl1 = ws.nsl1, nk1 = ws.nk1, nch = ws.nch, nsl2 = ws.nsl2, nk2 = ws.nk2, nds = ws.nds;
  auto steps_in = [&](int total, int part) __attribute__((always_inline)) { return ws.steps_in(total, part); };
  auto begin_step = [&]() __attribute__((always_inline)) { ws.begin_step(); };
  auto end_step = [&]() __attribute__((always_inline)) { ws.end_step(); };
  // transposing-read offsets of this lane (halves inside one staged step): rows 4 g .. + 3 and 8 + 4 g .. + 3 of the step, which
  // is the order in which an accumulator tile, rounded to fp16, supplies the contraction slots of the next product
  int troff[2], troffA[NTA];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int col = 64 * wave + 32 * j;
    troff[j] = (col >> 7) * (16 * 128) + tr_lane_off_swz(lane, (col & 127) >> 5) + 4 * g * 128;
  }
#pragma unroll
  for (int j = 0; j < NTA; ++j) {
    const int col = 32 * NTA * wave + 32 * j;
    troffA[j] = (col >> 7) * (16 * 128) + tr_lane_off_swz(lane, (col & 127) >> 5) + 4 * g * 128;
  }
  auto wfrag = [&](int off) __attribute__((always_inline)) {
    const _Float16* wt = &wbuf[0][0][0][0] + ws.buf * (kV2StepBytes / 2) + off;
    return tr_frag(wt, wt + 8 * 128);
  };

  f16v zacc[NSL][2][MT];                       // P1^T in step 1, Z^T in step 2: slab, column tile, token tile
  auto clear_z = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int sl = 0; sl < NSL; ++sl)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) zacc[sl][j][mt] = zero16();
  };
  // rank-space accumulators -> operand fragments of the next product (ranks below `n` only)
  auto publish_z = [&](int n) __attribute__((always_inline)) {
#pragma unroll
    for (int sl = 0; sl < NSL; ++sl)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int row0 = 512 * sl + 64 * wave + 32 * j;
        if (row0 < n) {
#pragma unroll
          for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
              h8 o;
#pragma unroll
              for (int i = 0; i < 8; ++i) o[i] = (_Float16)zacc[sl][j][mt][8 * s2 + i];
              pfr[(row0 / 16 + s2) * MT + mt][lane] = o;
            }
        }
      }
  };
  // one slab of a rank-space product: z += W^T[512 sl .., steps] . act
  auto rank_pass = [&](f16v (&z)[2][MT], int sl, int nsteps, int n, const h8* act) __attribute__((always_inline)) {
    const bool on0 = 512 * sl + 64 * wave < n, on1 = 512 * sl + 64 * wave + 32 < n;
    for (int ks = 0; ks < nsteps; ++ks) {
      begin_step();
      if (on0) {
        h8 af[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) af[mt] = act[(ks * MT + mt) * 64 + lane];
        const h8 b0 = wfrag(troff[0]);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) z[0][mt] = mfma32(b0, af[mt], z[0][mt]);
        if (on1) {
          const h8 b1 = wfrag(troff[1]);
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) z[1][mt] = mfma32(b1, af[mt], z[1][mt]);
        }
      }
      end_step();
    }
  };

  ws.start();

  // ================= step 1: P1^T = U_1^T X^T =================
  clear_z();
  for (int xs = 0; xs < nxs; ++xs) {
    const int kc = steps_in(D, xs);
    // X slab -> operand fragments: lane (token, g) of step ks holds columns 16 ks + 4 g + {0..3} and + 8 of its token
    for (int ks = wave; ks < kc; ks += 8) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int tok = tok0 + 32 * mt + l32;
        const size_t e = (size_t)tok * D + FC * xs + 16 * ks + 4 * g;
        f4v lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
        if (tok < T) { lo = load4(a.X, e, a.x_dt); hi = load4(a.X, e + 8, a.x_dt); }
        h8 o;
#pragma unroll
        for (int i = 0; i < 4; ++i) { o[i] = (_Float16)lo[i]; o[4 + i] = (_Float16)hi[i]; }
        gfr[ks * MT + mt][lane] = o;
      }
    }
    __syncthreads();
#pragma unroll
    for (int sl = 0; sl < NSL; ++sl)
      if (sl < nsl1) rank_pass(zacc[sl], sl, kc, r1, &gfr[0][0]);
  }
  publish_z(r1);
  clear_z();
  __syncthreads();

  // ================= step 2: chunks of F =================
  for (int ch = 0; ch < nch; ++ch) {
    f16v hacc[NTA][MT];
#pragma unroll
    for (int j = 0; j < NTA; ++j)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) hacc[j][mt] = zero16();
    const int f0 = FC * ch + 32 * NTA * wave;   // first feature of this wavefront
    bool onf[NTA];
#pragma unroll
    for (int j = 0; j < NTA; ++j) onf[j] = f0 + 32 * j < F;
    for (int ks = 0; ks < nk1; ++ks) {
      begin_step();
      if (onf[0]) {
        h8 af[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) af[mt] = pfr[ks * MT + mt][lane];
#pragma unroll
        for (int j = 0; j < NTA; ++j)
          if (onf[j]) {
            const h8 b = wfrag(troffA[j]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) hacc[j][mt] = mfma32(b, af[mt], hacc[j][mt]);
          }
      }
      end_step();
    }
    // + b_1, activation, fp16 -> operand fragments of the second product (the last barrier has retired every read of gfr)
#pragma unroll
    for (int j = 0; j < NTA; ++j)
      if (onf[j]) {
        f4v bias[4];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const int f = f0 + 32 * j + 8 * jj + 4 * g;
          bias[jj] = (a.b1 && f < F) ? load4(a.b1, f, a.w_dt) : f4v{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            h8 o;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
              const float x = hacc[j][mt][8 * s2 + i] + bias[2 * s2 + (i >> 2)][i & 3];
              const float y = a.act == 0 ? gelu_erf_f(x) : (a.act == 1 ? gelu_tanh_f(x) : fmaxf(x, 0.f));
              o[i] = (_Float16)y;
            }
            gfr[(2 * NTA * wave + 2 * j + s2) * MT + mt][lane] = o;
          }
      }
    __syncthreads();
    const int kc = steps_in(F, ch);
#pragma unroll
    for (int sl = 0; sl < NSL; ++sl)
      if (sl < nsl2) rank_pass(zacc[sl], sl, kc, r2, &gfr[0][0]);
  }

  // ================= step 3: out^T = V_2^T Z^T + b_2 =================
  publish_z(r2);
  __syncthreads();
  for (int ds = 0; ds < nds; ++ds) {
    f16v oacc[2][MT];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) oacc[j][mt] = zero16();
    const int n0 = 512 * ds + 64 * wave;
    const bool on0 = n0 < D, on1 = n0 + 32 < D;
    for (int ks = 0; ks < nk2; ++ks) {
      begin_step();
      if (on0) {
        h8 af[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) af[mt] = pfr[ks * MT + mt][lane];
        const h8 b0 = wfrag(troff[0]);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) oacc[0][mt] = mfma32(b0, af[mt], oacc[0][mt]);
        if (on1) {
          const h8 b1 = wfrag(troff[1]);
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) oacc[1][mt] = mfma32(b1, af[mt], oacc[1][mt]);
        }
      }
      end_step();
    }
#pragma unroll
    for (int j = 0; j < 2; ++j)
      if (n0 + 32 * j < D) {
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const int n = n0 + 32 * j + 8 * jj + 4 * g;
          const f4v b = a.b2 ? load4(a.b2, n, a.w_dt) : f4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            const int tok = tok0 + 32 * mt + l32;
            f4v y;
#pragma unroll
            for (int e = 0; e < 4; ++e) y[e] = oacc[j][mt][4 * jj + e] + b[e];
            if (tok < T) store4(a.out, (size_t)tok * D + n, y, a.out_dt);
          }
        }
      }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the two requests past the end have landed before the workgroup retires
}

}  // namespace

bool ffn_v2_supported(int D, int F, int r1, int r2) {
  return D % 32 == 0 && F % 16 == 0 && r1 % 16 == 0 && r2 % 16 == 0 && r1 <= 1024 && r2 <= 1024;
}

hipError_t launch_ffn_v2(const FfnV2Args& a, hipStream_t s) {
  if (!ffn_v2_supported(a.D, a.F, a.r1, a.r2) || a.T <= 0) return hipErrorInvalidValue;
  // 64 tokens per workgroup halve the weight traffic; they need both ranks <= 512 and enough tokens to fill the chip
  if (a.r1 <= 512 && a.r2 <= 512 && (a.T + 63) / 64 >= 200)
    hipLaunchKernelGGL(ffn_v2_kernel<2>, dim3((a.T + 63) / 64), dim3(kV2Threads), 0, s, a);
  else
    hipLaunchKernelGGL(ffn_v2_kernel<1>, dim3((a.T + 31) / 32), dim3(kV2Threads), 0, s, a);
  return hipGetLastError();
}

}  // namespace fsvd
