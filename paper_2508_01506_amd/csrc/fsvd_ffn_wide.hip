// Fused FFN core (Alg. 2, the on-chip loops) for prepacked weights and wide rank slices:
//   Z[T, r2] = phi(P1[T, r1] V_1[r1, F] + b_1) U_2[F, r2],  hidden activation only on chip.
//
// Same decomposition as ffn_core_kernel (one workgroup = 64 tokens x one slice of up to 1024 output ranks x one part of
// F, accumulator Z^T in registers over the whole sweep), different use of the eight wavefronts: all of them compute in
// every stage and all of them request tiles, two per SIMD so that one wavefront's operand reads run under the other's
// MFMAs.  F is swept in chunks of 256 features:
//   phase A  Y^T[256 f, 64 tok] = V_1[:, chunk]^T P1^T in stages of 64 ranks.  Wavefront (rho, w) owns features
//            64 w .. 64 w + 63 (a 2 x 2 block of 32 x 32 tiles: every operand read from LDS feeds two MFMAs) and the
//            contraction steps 2 rho, 2 rho + 1 of each stage, so the two wavefronts of a SIMD split the contraction;
//            at the end of the chunk the pair exchanges halves of its partial sums through LDS (fp32), and each
//            wavefront adds b_1, applies phi to 32 features x 64 tokens and publishes them as fp16 MFMA operands;
//   phase B  Z^T[rank, tok] += U_2[chunk, :]^T Y^T in stages of 64 features x 256 ranks; wavefront (rho, w) owns
//            ranks 256 p + 128 rho + 32 w .. + 31 of every 256-rank group p of the slice; the activated operands of
//            the current 64 features stay in registers over the groups.
// Every stage is one ring slot of LDS (three slots): weight pieces are halves of 128 x 128 tile images and the P1
// pieces are fragment-major blocks, both copied straight into LDS by loads that bypass the registers, five (phase A)
// or four (phase B) per wavefront and stage, requested three stages ahead.  One workgroup barrier per stage; the
// operands of stage i + 1 are read from LDS while the MFMAs of stage i run.
#include "fsvd_common.h"
#include "fsvd_kernels.h"

namespace fsvd {

namespace {

constexpr int kBT = 64;                       // tokens per workgroup
constexpr int kBF = 256;                      // features per chunk
constexpr int kRowH = 128;                    // halves per row of a tile image
constexpr int kPieceBytes = 16384;            // half a tile image: 64 rows
constexpr int kStageW = 2 * kPieceBytes;      // weight bytes per stage
constexpr int kStageP = 8192;                 // P1 bytes per phase-A stage: 64 ranks x 64 tokens
constexpr int kSlot = kStageW + kStageP;
constexpr int kGBytes = 32768;                // activated chunk as fp16 operands; before that the fp32 exchange buffer

typedef const __attribute__((address_space(4))) uint32_t* const_u32_ptr;   // read through the scalar unit

__device__ __forceinline__ void lds_wait_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int NP>
__global__ void __launch_bounds__(512, 1) ffn_core_wide_kernel(FfnCoreArgs a, int nslices, int fsplit) {
  __shared__ __attribute__((aligned(1024))) unsigned char ring[3][kSlot];
  __shared__ __attribute__((aligned(1024))) unsigned char gx[kGBytes];

  const int tid = threadIdx.x;
  const int lane = tid & 63, l32 = lane & 31, g = lane >> 5;
  const int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int rho = wave8 >> 2, w = wave8 & 3;
  const int wg = xcd_tile(blockIdx.x, gridDim.x);
  const int slice = wg % nslices;
  const int ntile = (a.T + kBT - 1) / kBT;
  const int tb = (wg / nslices) % ntile;
  const int fs = wg / (nslices * ntile);
  const int t0 = tb * kBT;
  const int s0 = slice * 256 * NP;
  const int r1 = a.r1, r2 = a.r2, F = a.F, T = a.T;
  const int nA = (r1 + 63) / 64;                             // phase-A stages per chunk = 64-rank pieces of P1
  const int pch = nA, ptiles = (T + 31) / 32;
  const int ntF = (F + 127) / 128, ntR2 = (r2 + 127) / 128;
  const int nch_all = (F + kBF - 1) / kBF;
  const int cps = (nch_all + fsplit - 1) / fsplit;
  const int c_begin = fs * cps;
  const int c_end = (c_begin + cps < nch_all) ? c_begin + cps : nch_all;
  const int per_chunk = nA + 4 * NP;
  // The workgroups of one XCD (every eighth one) sweep the same weight tiles at about the same time.  Each starts the
  // contraction over r1 at a different 64-rank block, so that at any moment they ask the L2 for different tiles (many
  // distinct misses in flight instead of the same miss many times) and find the others' tiles there later on.  The
  // order of the fp32 sums depends on the workgroup index only: results stay reproducible.
  const int a_rot = (int)(((blockIdx.x >> 3) & 31) * (unsigned)nA / 32u);

  // ---------------------------------------------------------------- tile requests (every wavefront its share)
  const u4 rV1 = lds_dma_rsrc(uniform_ptr(a.V1), (unsigned)tiled_bytes(r1, F));
  const u4 rU2 = lds_dma_rsrc(uniform_ptr(a.U2), (unsigned)tiled_bytes(F, r2));
  const u4 rP = lds_dma_rsrc(uniform_ptr(a.P1), (unsigned)fm_bytes(T, r1));
  const int voff = lane * 16;
  const unsigned ring0 = lds_addr_of(&ring[0][0]);
  int rq_c = c_begin, rq_j = 0, rq_slot = 0;
  bool last_isA = true;
  // Requests past the last stage of this workgroup re-read valid tiles (clamped indices): they land in a slot nobody
  // reads any more.  Indices past the padded tensors are clamped as well; what such a tile contributes is discarded
  // (features >= F are zeroed when the chunk is published, ranks >= r2 are not written).
  auto request_next = [&]() {
    const int c = rq_c < nch_all ? rq_c : nch_all - 1;
    const unsigned dst = ring0 + rq_slot * kSlot;
    if (rq_j < nA) {
      int ra = rq_j + a_rot;           // this workgroup's rotation of the contraction order
      ra = ra >= nA ? ra - nA : ra;
      const int kt = ra >> 1, half = ra & 1;
#pragma unroll
      for (int n = 0; n < 4; ++n) {
        const int i = wave8 + 8 * n, j = n >> 1, sub = wave8 + 8 * (n & 1);
        int nt = 2 * c + j;
        nt = nt < ntF ? nt : ntF - 1;
        lds_dma16(rV1, dst + i * 1024, voff, (kt * ntF + nt) * kTileImageBytes + half * kPieceBytes + sub * 1024);
      }
      int tile = (t0 >> 5) + (wave8 >> 2);
      tile = tile < ptiles ? tile : ptiles - 1;
      lds_dma16(rP, dst + kStageW + wave8 * 1024, voff, (tile * pch + ra) * kFmChunkBytes + (wave8 & 3) * 1024);
      last_isA = true;
    } else {
      const int jb = rq_j - nA, q = jb / NP, p = jb - q * NP;
      int ft = 2 * c + (q >> 1);
      ft = ft < ntF ? ft : ntF - 1;
#pragma unroll
      for (int n = 0; n < 4; ++n) {
        const int i = wave8 + 8 * n, j = n >> 1, sub = wave8 + 8 * (n & 1);
        int rt = (s0 >> 7) + 2 * p + j;
        rt = rt < ntR2 ? rt : ntR2 - 1;
        lds_dma16(rU2, dst + i * 1024, voff, (ft * ntR2 + rt) * kTileImageBytes + (q & 1) * kPieceBytes + sub * 1024);
      }
      last_isA = false;
    }
    if (++rq_j == per_chunk) { rq_j = 0; ++rq_c; }
    rq_slot = rq_slot == 2 ? 0 : rq_slot + 1;
  };
  // Start of stage i: everything this wavefront read from slot i (the stage's operands, fetched during stage i - 1) has
  // arrived and its requests for stage i + 1 have landed (only those for stage i + 2, the most recent ones, may still be
  // in flight: loads complete in issue order); after the barrier that holds for all wavefronts, so slot i is free for
  // stage i + 3 and slot i + 1 may be read.
  auto stage_sync = [&]() {
    if (last_isA) lds_dma_wait_barrier<5>();
    else lds_dma_wait_barrier<4>();
    request_next();
  };

  // ---------------------------------------------------------------- operand reads
  const int trA0 = tr_lane_off_swz(lane, 2 * (w & 1)) + 32 * g * kRowH;       // phase A: features 64 w + 0..31
  const int trA1 = tr_lane_off_swz(lane, 2 * (w & 1) + 1) + 32 * g * kRowH;   //          features 64 w + 32..63
  const int trB = tr_lane_off_swz(lane, w) + 4 * g * kRowH;                   // phase B: ranks 32 w .. of the wavefront's piece
  h8 aw[2][2], ap[2][2];      // phase A operands [step][feature tile], [step][token tile]
  h8 bw[4];                   // phase B weight operands, one per 16-feature step
  h8 gq[4][2];                // activated operands of the current 64 features [step][token tile]
  auto load_a = [&](const unsigned char* slot, int k) {
    const int kk = 2 * rho + k;
    const _Float16* wb = (const _Float16*)slot + (w >> 1) * (kPieceBytes / 2) + 8 * kk * kRowH;
    aw[k][0] = tr_frag(wb + trA0, wb + trA0 + 4 * kRowH);
    aw[k][1] = tr_frag(wb + trA1, wb + trA1 + 4 * kRowH);
    const h8* pb = (const h8*)(slot + kStageW);
    ap[k][0] = pb[kk * 64 + lane];
    ap[k][1] = pb[(4 + kk) * 64 + lane];
  };
  auto load_b = [&](const unsigned char* slot, int f) {
    const _Float16* wb = (const _Float16*)slot + rho * (kPieceBytes / 2) + trB + 16 * f * kRowH;
    return tr_frag(wb, wb + 8 * kRowH);
  };
  auto load_g = [&](int q) {
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) gq[f][tt] = ((const h8*)gx)[(((2 * q + (f >> 1)) * 2 + (f & 1)) * 2 + tt) * 64 + lane];
  };

  f16v z[NP][2], y[2][2];
#pragma unroll
  for (int p = 0; p < NP; ++p) { z[p][0] = zero16(); z[p][1] = zero16(); }

  // End of phase A for one chunk: the pair (rho = 0, 1) of a SIMD holds partial sums over complementary contraction
  // steps of the same 64 features.  `send` goes to the partner, the partner's half is added to `keep`; then bias,
  // activation, fp16, publish as operands of phase B (features 32 ft .., ft = 2 w + rho).
  auto finish_chunk = [&](f16v (&keep)[2], f16v (&send)[2], int c) {
    f4v* xb = (f4v*)gx;
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        f4v v = {send[tt][4 * j], send[tt][4 * j + 1], send[tt][4 * j + 2], send[tt][4 * j + 3]};
        xb[(wave8 * 4 + j) * 64 + lane] = v;
      }
      lds_wait_barrier();
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const f4v v = xb[((wave8 ^ 4) * 4 + j) * 64 + lane];
#pragma unroll
        for (int i = 0; i < 4; ++i) keep[tt][4 * j + i] += v[i];
        if (j == 1) __builtin_amdgcn_sched_barrier(0);   // two reads in flight at a time are enough here
      }
      lds_wait_barrier();      // the buffer is rewritten next (second half, then the published chunk)
    }
    const int ft = 2 * w + rho;
    const int f0 = c * kBF + 32 * ft;
    // b_1 of the wavefront's 32 features through the scalar unit (its loads are not counted with the tile requests)
    uint32_t bwd[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) bwd[i] = 0u;
    if (a.b1 != nullptr && f0 < F) {
      const_u32_ptr bp = (const_u32_ptr)(uintptr_t)((const char*)uniform_ptr(a.b1) + (size_t)f0 * 2);
#pragma unroll
      for (int i = 0; i < 8; ++i) bwd[i] = bp[i];
      if (f0 + 16 < F) {
#pragma unroll
        for (int i = 0; i < 8; ++i) bwd[8 + i] = bp[8 + i];
      }
    }
    float bias[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {     // accumulator v of this lane: feature row 8 (v / 4) + 4 g + v % 4
      const int d0 = 4 * (v >> 2) + ((v & 3) >> 1);
      const uint32_t word = g ? bwd[d0 + 2] : bwd[d0];
      const uint32_t bits = (v & 1) ? (word >> 16) : (word & 0xffffu);
      bias[v] = a.w_dt == DT_BF16 ? __uint_as_float(bits << 16) : (float)__builtin_bit_cast(_Float16, (uint16_t)bits);
    }
    const bool ragged = f0 + 32 > F;   // features >= F: the weight tiles behind them are re-read ones, not zeros
    auto publish = [&](auto phi) {
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          h8 r;
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const int v = 8 * t + i;
            float x = phi(keep[tt][v] + bias[v]);
            if (ragged && f0 + 8 * (v >> 2) + 4 * g + (v & 3) >= F) x = 0.f;
            r[i] = (_Float16)x;
          }
          ((h8*)gx)[((ft * 2 + t) * 2 + tt) * 64 + lane] = r;
          __builtin_amdgcn_sched_barrier(0);   // one group of eight at a time: interleaving all 32 evaluations costs registers
        }
    };
    if (a.act == 0) publish([](float x) { return gelu_erf_f(x); });
    else if (a.act == 1) publish([](float x) { return gelu_tanh_f(x); });
    else publish([](float x) { return fmaxf(x, 0.f); });
    lds_wait_barrier();
  };

  // ---------------------------------------------------------------- main loop
  int sb = 0;                                   // slot of the stage about to run
  auto nxt = [](int s) { return s == 2 ? 0 : s + 1; };
  if (c_begin < c_end) {
    request_next();
    request_next();
    if (last_isA) lds_dma_wait_barrier<5>();    // stage 0 has landed
    else lds_dma_wait_barrier<4>();
    load_a(ring[0], 0);
    load_a(ring[0], 1);
    request_next();
  }
  // Operand registers are refilled unconditionally, also where the next stage is of the other kind or does not exist
  // (the slot read then holds some other landed tile and the values are never used): a conditional refill would keep
  // the previous contents alive across the other phase and cost their registers there.
  for (int c = c_begin; c < c_end; ++c) {
#pragma unroll
    for (int i = 0; i < 2; ++i) { y[i][0] = zero16(); y[i][1] = zero16(); }   // (not live during phase B)
    for (int s = 0; s < nA; ++s) {
      stage_sync();
      const unsigned char* nx = ring[nxt(sb)];
#pragma unroll
      for (int k = 0; k < 2; ++k) {
#pragma unroll
        for (int fi = 0; fi < 2; ++fi)
#pragma unroll
          for (int tt = 0; tt < 2; ++tt) y[fi][tt] = mfma32(aw[k][fi], ap[k][tt], y[fi][tt]);   // rows features, cols tokens
        __builtin_amdgcn_sched_barrier(0);    // the refill reuses the registers the MFMAs above have just read
        load_a(nx, k);
        __builtin_amdgcn_sched_barrier(0);
      }
      sb = nxt(sb);
    }
    if (rho == 0) finish_chunk(y[0], y[1], c);
    else finish_chunk(y[1], y[0], c);
    // the first stage of phase B landed before the last barrier of phase A
#pragma unroll
    for (int f = 0; f < 4; ++f) bw[f] = load_b(ring[sb], f);
    load_g(0);
    for (int q = 0; q < 4; ++q) {
#pragma unroll
      for (int p = 0; p < NP; ++p) {
        stage_sync();
        const unsigned char* nx = ring[nxt(sb)];
        const bool active = s0 + 256 * p + 128 * rho < r2;
#pragma unroll
        for (int f = 0; f < 4; ++f) {
          if (active) {
            z[p][0] = mfma32(bw[f], gq[f][0], z[p][0]);     // rows ranks, cols tokens
            z[p][1] = mfma32(bw[f], gq[f][1], z[p][1]);
          }
          bw[f] = load_b(nx, f);
        }
        if (p == NP - 1) load_g(q < 3 ? q + 1 : 3);
        sb = nxt(sb);
      }
    }
    // the next chunk's first stage (if any) landed before the last barrier
    load_a(ring[sb], 0);
    load_a(ring[sb], 1);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // nothing may still be writing LDS when the workgroup ends

  // ---------------------------------------------------------------- write Z (or this part's fp32 partial sums)
  const int zch = (r2 + 63) / 64;
#pragma unroll
  for (int tt = 0; tt < 2; ++tt) {
    const int tok = t0 + 32 * tt + l32;
    if (tok >= T) continue;
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const int r = s0 + 256 * p + 128 * rho + 32 * w + 8 * jj + 4 * g;
        if (r < zch * 64) {        // ranks r2 .. 64 zch - 1 are written as zeros (fragment-major padding)
          if (fsplit == 1) {
            const size_t unit = ((size_t)((tok >> 5) * zch + (r >> 6)) * 4 + ((r >> 3) & 3)) * 64 + ((r >> 5) & 1) * 32 + (tok & 31);
            h4 o;
#pragma unroll
            for (int i = 0; i < 4; ++i) o[i] = (_Float16)z[p][tt][4 * jj + i];
            *(h4*)((_Float16*)a.Z + unit * 8 + 4 * ((r >> 2) & 1)) = o;
          } else {
            f4v o;
#pragma unroll
            for (int i = 0; i < 4; ++i) o[i] = z[p][tt][4 * jj + i];
            *(f4v*)(a.Zpart + (((size_t)fs * (zch * 16) + (r >> 2)) * T + tok) * 4) = o;
          }
        }
      }
  }
}

}  // namespace

hipError_t launch_ffn_core_wide(const FfnCoreArgs& a, const FfnCorePlan& pl, hipStream_t s) {
  const dim3 grid(((a.T + kBT - 1) / kBT) * pl.nslices * pl.fsplit), block(512);
  switch (pl.wide) {
    case 1: hipLaunchKernelGGL((ffn_core_wide_kernel<1>), grid, block, 0, s, a, pl.nslices, pl.fsplit); break;
    case 2: hipLaunchKernelGGL((ffn_core_wide_kernel<2>), grid, block, 0, s, a, pl.nslices, pl.fsplit); break;
    case 3: hipLaunchKernelGGL((ffn_core_wide_kernel<3>), grid, block, 0, s, a, pl.nslices, pl.fsplit); break;
    case 4: hipLaunchKernelGGL((ffn_core_wide_kernel<4>), grid, block, 0, s, a, pl.nslices, pl.fsplit); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace fsvd
