// Fused FFN core (Alg. 2, the on-chip loops): Z[T, r2] = phi(P1[T, r1] V_1[r1, F] + b_1) U_2[F, r2].
// The hidden activation phi(...) [T, F] exists only as 128-wide slabs in registers / LDS.
//
// One workgroup owns 64 tokens, one slice of at most 1024 output ranks and one part of F; its 8 wavefronts
// have two roles.
//   Compute wavefronts (4, one per SIMD) keep the accumulator Z^T [up to 512 ranks, 64 tokens] in registers for
//   the whole sweep over F.  Per 128-wide chunk of F:
//     phase A  Y^T[128 f, 64 tok] = V_1[:, chunk]^T P1^T, contraction over r1 in 128-wide stages; wavefront w
//              computes features 32*w.., adds b_1, applies phi, rounds to fp16 and publishes the result to all
//              wavefronts through LDS in MFMA operand order;
//     phase B  Z^T[128*s + 32*w.., 64 tok] += U_2[chunk, :]^T Y^T, one 128-rank sub-tile s per stage.
//   Loader wavefronts (4) run the same sequence of stages one tile ahead: every weight tile (128 contraction rows
//   x 128 output columns) is copied as it lies in memory into a double-buffered LDS tile (bf16 widened to fp16 on
//   the way) and read back by the compute wavefronts with the LDS's transposing read; while tile i is in use, tile
//   i+1 (requested one stage earlier) is stored and tile i+2 is requested, pass by pass.  The P1 tiles of phase A
//   (fragment-major, contiguous) travel the same way through a second double buffer.  One barrier per stage.
//   When the slice is wider than 512 ranks the loaders' otherwise idle registers hold the accumulators of the
//   remaining sub-tiles and they issue those sub-tiles' MFMAs between their staging passes, so one pass of phase A
//   serves up to 1024 ranks.
// Slices of r2 beyond that are separate workgroups (phase A is recomputed per slice).  When there are fewer
// workgroups than compute units the sum over F is split across workgroups: each writes fp32 partial sums and a
// second kernel adds them in a fixed order.  ffn_core_plan() picks the shape on the host.
#include "fsvd_common.h"
#include "fsvd_kernels.h"

#include <stdlib.h>

namespace fsvd {

namespace {

constexpr int kFfnBT = 64;                  // tokens per workgroup
constexpr int kFfnBF = 128;                 // F chunk
constexpr int kTile = 128;                  // weight tile edge
constexpr int kTileRow = wtile_stride(kTile);   // halves per LDS tile row

// One output tile of a wavefront's accumulators: ranks [rbase + 128 s + 32 wave ..) of tokens t0.. -> either the final
// fragment-major fp16 Z (4 consecutive ranks per 8-byte store) or, when F is split across workgroups, this
// workgroup's fp32 partial sums, laid out [split][rank / 4][token][4] so that a wavefront writes 512-byte runs.
template <int N>
__device__ __forceinline__ void write_z(const f16v (&z)[N][2], const FfnCoreArgs& a, int fsplit, int fs, int t0, int rbase,
                                        int rlimit, int wave, int l32, int g) {
  const int T = a.T, zch = (a.r2 + 63) / 64;
#pragma unroll
  for (int tt = 0; tt < 2; ++tt) {
    const int tok = t0 + 32 * tt + l32;
    if (tok >= T) continue;
#pragma unroll
    for (int s = 0; s < N; ++s)
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const int r = rbase + s * kTile + 32 * wave + 8 * jj + 4 * g;
        if (r < rlimit && r < zch * 64) {   // ranks r2 .. 64*zch-1 are written as zeros (FM padding)
          if (fsplit == 1) {
            const size_t unit = ((size_t)((tok >> 5) * zch + (r >> 6)) * 4 + ((r >> 3) & 3)) * 64 + ((r >> 5) & 1) * 32 + (tok & 31);
            h4 o;
#pragma unroll
            for (int i = 0; i < 4; ++i) o[i] = (_Float16)z[s][tt][4 * jj + i];
            *(h4*)((_Float16*)a.Z + unit * 8 + 4 * ((r >> 2) & 1)) = o;
          } else {
            f4v o;
#pragma unroll
            for (int i = 0; i < 4; ++i) o[i] = z[s][tt][4 * jj + i];
            *(f4v*)(a.Zpart + (((size_t)fs * (zch * 16) + (r >> 2)) * T + tok) * 4) = o;
          }
        }
      }
  }
}

// NS: 128-rank sub-tiles accumulated by the compute wavefronts, NS2: further sub-tiles accumulated by the loader
// wavefronts (their registers are otherwise idle), so that one workgroup covers up to 1024 output ranks with a single
// pass of phase A.
// WT: DT_F16 / DT_BF16 = row-major weights of that type, staged through registers into padded LDS rows (two buffers);
// kWtTiled = weights prepacked as fp16 tile images (see fsvd_common.h), copied by the loaders straight from memory into
// LDS without passing through registers (three buffers, requests two tiles ahead).
template <int NS, int NS2, int WT>
__global__ void __launch_bounds__(512, 1) ffn_core_kernel(FfnCoreArgs a, int nslices, int slice_w, int fsplit) {
  constexpr bool PK = (WT == kWtTiled);
  constexpr int NB = PK ? 3 : 2;                           // LDS buffers per stream
  constexpr int kRow = PK ? kTile : kTileRow;              // halves per LDS tile row
  __shared__ __attribute__((aligned(1024))) _Float16 wt_lds[NB][kTile * kRow];
  __shared__ __attribute__((aligned(1024))) h8 ptile[NB][16][64];    // [buffer][(token tile * 2 + hh) * 4 + kk][lane]
  __shared__ __attribute__((aligned(16))) h8 gtile[4][2][2][64];     // [f tile][t][token tile][lane]

  const int tid = threadIdx.x;
  const int lane = tid & 63, l32 = lane & 31, g = lane >> 5;
  const int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps everything derived from it in scalar registers
  const int wave = wave8 & 3;                                    // index inside the role
  const bool loader = wave8 >= 4;
  // The slices of one token tile re-read the same P1 block once per chunk of F: keep them (and neighbouring token
  // tiles) on one XCD so that those re-reads hit its L2 instead of each XCD's L2 cycling through all of P1.
  const int wg = xcd_tile(blockIdx.x, gridDim.x);
  const int slice = wg % nslices;
  const int ntile = (a.T + kFfnBT - 1) / kFfnBT;
  const int tb = (wg / nslices) % ntile;
  const int fs = wg / (nslices * ntile);                        // which part of F this workgroup sums over
  const int t0 = tb * kFfnBT;
  const int s0 = slice * slice_w;                               // first output rank of this slice
  const int r1 = a.r1, F = a.F, r2 = a.r2, T = a.T;
  const int s_end = (s0 + slice_w < r2) ? s0 + slice_w : r2;
  const int nA = (r1 + kTile - 1) / kTile;
  const int nchunks_all = (F + kFfnBF - 1) / kFfnBF;
  const int cps = (nchunks_all + fsplit - 1) / fsplit;
  const int c_begin = fs * cps;
  const int nchunks = (c_begin + cps < nchunks_all) ? c_begin + cps : nchunks_all;   // this workgroup: chunks c_begin .. nchunks-1
  const int per_chunk = nA + NS + NS2;                          // tiles per chunk: nA of V_1, then NS + NS2 of U_2
  const int pch = (r1 + 63) / 64, zch = (r2 + 63) / 64;

  // LDS buffers rotate: the tile in use sits in buffer `it % NB`
  auto nxt = [](int b) { return b + 1 == NB ? 0 : b + 1; };
  // per-lane part of the transposing reads of a weight tile (columns 32 * wave ..)
  const int trl = PK ? tr_lane_off_swz(lane, wave) : tr_lane_off(lane, kRow) + 32 * wave;
  const int trA = trl + 32 * g * kRow;   // phase A: k rows 32 g + 8 kk + 0..7
  const int trB = trl + 4 * g * kRow;    // phase B: k rows 16 fs + 4 g + {0..3, 8..11}

  if (loader) {
    // sub-tiles NS .. NS+NS2-1 of phase B run on the loader wavefronts; `between(f)` is called after the MFMAs of step f
    f16v z2[NS2 > 0 ? NS2 : 1][2];
#pragma unroll
    for (int s = 0; s < (NS2 > 0 ? NS2 : 1); ++s) { z2[s][0] = zero16(); z2[s][1] = zero16(); }
    auto stage_b2 = [&](const _Float16* wb, f16v (&zs)[2], bool active, auto between) {
      h8 wf = tr_frag(wb + trB, wb + trB + 8 * kRow);
      h8 g0 = gtile[0][0][0][lane], g1 = gtile[0][0][1][lane];
#pragma unroll
      for (int f = 0; f < 8; ++f) {
        h8 wf_next = wf, n0 = g0, n1 = g1;
        if (f < 7) {
          const _Float16* q = wb + trB + 16 * (f + 1) * kRow;
          wf_next = tr_frag(q, q + 8 * kRow);
          n0 = gtile[(f + 1) >> 1][(f + 1) & 1][0][lane];
          n1 = gtile[(f + 1) >> 1][(f + 1) & 1][1][lane];
        }
        if (active) {
          zs[0] = mfma32(wf, g0, zs[0]);
          zs[1] = mfma32(wf, g1, zs[1]);
        }
        between(f);
        wf = wf_next; g0 = n0; g1 = n1;
      }
    };

    if constexpr (PK) {
      // =====================================================================================================
      // Loader wavefronts, prepacked weights.  A tile image is 32 KiB that go to LDS byte for byte: wavefront w
      // moves the 1 KiB pieces 4 p + w (p = 0..7) with loads that write LDS directly, so a tile costs 8
      // instructions per wavefront and no registers.  Tile i+2 is requested while tile i is in use (three
      // buffers); loads complete in order, so waiting until only the requests of this stage are outstanding
      // means tile i+1 has landed.  The P1 tiles of phase A (16 KiB, fragment-major = LDS order) travel the same way.
      // Nothing here depends on out-of-range reads: tile images are zero-padded to whole tiles, requests past the
      // end of the stream re-read the last tile, and a rank piece past r1 re-reads the last valid piece (its
      // weight rows are zero).
      // =====================================================================================================
      const int ntF = (F + kTile - 1) / kTile, ntR2 = (r2 + kTile - 1) / kTile;
      const char* const pV1 = uniform_ptr(a.V1);
      const char* const pU2 = uniform_ptr(a.U2);
      const int voff = lane * 16;
      const unsigned lds_w0 = lds_addr_of(&wt_lds[0][0]), lds_p0 = lds_addr_of(&ptile[0][0][0]);
      auto request_tile = [&](int buf, int c, int j) {
        c = c < nchunks ? c : nchunks - 1;
        const bool isA = j < nA;
        int nt2 = (s0 >> 7) + (j - nA);
        nt2 = nt2 < ntR2 ? nt2 : ntR2 - 1;
        const long long tile = isA ? ((long long)j * ntF + c) : ((long long)c * ntR2 + nt2);
        const unsigned long long sel = isA ? 1 : 0;
        const unsigned long long base = (unsigned long long)pU2 + ((unsigned long long)pV1 - (unsigned long long)pU2) * sel;
        const u4 r = lds_dma_rsrc((const void*)(base + (unsigned long long)tile * kTileImageBytes), kTileImageBytes);
        const unsigned dst = lds_w0 + buf * kTileImageBytes + wave * 1024;
#pragma unroll
        for (int p = 0; p < 8; ++p) lds_dma16(r, dst + p * 4096, voff, (4 * p + wave) * 1024);
      };
      const int ptiles = (T + 31) / 32;
      const u4 rP = lds_dma_rsrc(uniform_ptr(a.P1), (unsigned)fm_bytes(T, r1));
      auto request_p = [&](int buf, int ra) {
        const unsigned dst = lds_p0 + buf * 16384 + wave * 1024;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          int piece = 2 * ra + (j & 1), tt = (t0 >> 5) + (j >> 1);
          piece = piece < pch ? piece : pch - 1;
          tt = tt < ptiles ? tt : ptiles - 1;
          lds_dma16(rP, dst + j * 4096, voff, (tt * pch + piece) * kFmChunkBytes + wave * 1024);
        }
      };
      auto request2 = [&](int buf, int c, int j) {          // tile two ahead of (c, j)
        int c2 = c, j2 = j + 2;
        if (j2 >= per_chunk) { j2 -= per_chunk; ++c2; }
        request_tile(buf, c2, j2);
      };
      // prologue: tiles 0 and 1 and the P1 tiles of the first two stages
      request_tile(0, c_begin, 0);
      request_p(0, 0);
      request_tile(1, c_begin, 1);                          // per_chunk >= 2
      request_p(1, 1 % nA);
      lds_dma_wait_barrier<12>();                           // tile 0 and its P1 tile are in LDS
      int wb = 0, pb = 0;                                   // buffers of the tile / P1 tile in use
      for (int c = c_begin; c < nchunks; ++c) {
        for (int ra = 0; ra < nA; ++ra) {
          request2(nxt(nxt(wb)), c, ra);
          request_p(nxt(nxt(pb)), (ra + 2) % nA);
          lds_dma_wait_barrier<12>();                       // everything requested before this stage has landed
          wb = nxt(wb); pb = nxt(pb);
        }
        for (int s = 0; s < NS; ++s) {
          request2(nxt(nxt(wb)), c, nA + s);
          lds_dma_wait_barrier<8>();
          wb = nxt(wb);
        }
        if constexpr (NS2 > 0) {
          // these wavefronts stage nothing through registers, so the chunk's activation operands fit in them (as in
          // the compute wavefronts): one LDS read of the weight fragment per step instead of three
          h8 gq2[8][2];
#pragma unroll
          for (int f = 0; f < 8; ++f)
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) gq2[f][tt] = gtile[f >> 1][f & 1][tt][lane];
#pragma unroll
          for (int s = 0; s < NS2; ++s) {
            request2(nxt(nxt(wb)), c, nA + NS + s);
            const _Float16* w2 = wt_lds[wb];
            const bool active = s0 + (NS + s) * kTile < s_end;
            h8 wf = tr_frag(w2 + trB, w2 + trB + 8 * kRow);
#pragma unroll
            for (int f = 0; f < 8; ++f) {
              h8 wf_next = wf;
              if (f < 7) {
                const _Float16* q = w2 + trB + 16 * (f + 1) * kRow;
                wf_next = tr_frag(q, q + 8 * kRow);
              }
              if (active) {
                z2[s][0] = mfma32(wf, gq2[f][0], z2[s][0]);
                z2[s][1] = mfma32(wf, gq2[f][1], z2[s][1]);
              }
              wf = wf_next;
            }
            lds_dma_wait_barrier<8>();
            wb = nxt(wb);
          }
        }
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // nothing may still be writing LDS when the workgroup ends
    } else {
    // =====================================================================================================
    // Loader wavefronts, row-major weights: tile i+1 of the weight stream (requested one stage ago) is converted
    // and written to the LDS buffer the compute wavefronts will read next, tile i+2 is requested from global
    // memory; the P1 tiles of phase A travel the same way.
    // Tile (c, j): j < nA -> V_1 rows 128 j.., columns f of chunk c; j >= nA -> U_2 rows f of chunk c,
    // columns s0 + 128 (j - nA)..   Thread -> tile row s_r (+ 16 per pass), 8 columns from s_c.
    // =====================================================================================================
    const int lt = tid & 255;
    const int s_r = lt >> 4, s_c = 8 * (lt & 15);
    const long long p_total = (long long)fm_bytes(T, r1);
    const long long v1_total = (long long)r1 * F * 2, u2_total = (long long)F * r2 * 2;
    const char* const pV1 = uniform_ptr(a.V1);
    const char* const pU2 = uniform_ptr(a.U2);
    u4 w_raw[8], p_raw[4];
    const char* src_base = nullptr;   // source of the tile currently being requested (two ahead of the tile in use)
    int src_left = 0;
    unsigned src_v0 = 0, src_ld = 0;
    auto tile_src = [&](int c, int j) {
      const bool isA = j < nA;
      const int ld = isA ? F : r2;
      const long long off = isA ? ((long long)j * kTile * F + c * kFfnBF) : ((long long)c * kFfnBF * r2 + s0 + (j - nA) * kTile);
      const int cols = isA ? (F - c * kFfnBF) : (s_end - s0 - (j - nA) * kTile);      // valid columns of this tile
      // branch-free scalar arithmetic (a chain of selects over kernel arguments would be turned into a table in scratch)
      const long long sel = isA ? 1 : 0, live = (c < nchunks) ? 1 : 0;
      long long left = (u2_total + (v1_total - u2_total) * sel) * live - off * 2;       // past the last tile: nothing
      left = left < 0 ? 0 : left;
      const unsigned long long pb = (unsigned long long)pU2 + ((unsigned long long)pV1 - (unsigned long long)pU2) * (unsigned long long)sel;
      src_base = (const char*)pb + (left > 0 ? off * 2 : 0);
      src_left = (int)left;
      src_v0 = (s_c < cols) ? (unsigned)(s_r * ld + s_c) * 2u : (unsigned)kOobOffset;
      src_ld = (unsigned)ld;
    };
    auto issue_pass = [&](int p) {      // rows past the end of the tensor: 0
      const rsrc_t r = __builtin_amdgcn_make_buffer_rsrc((void*)src_base, 0, src_left, 0x00020000);
      w_raw[p] = buf_load16(r, (int)(src_v0 + (unsigned)(32 * p) * src_ld));
    };
    auto commit_pass = [&](int pb, int p) { stage_store16<WT>(&wt_lds[pb][(s_r + 16 * p) * kRow + s_c], w_raw[p]); };
    // P1 tile of phase-A stage ra: four 4 KiB fragment-major blocks (token tile tt, 64-wide piece 2 ra + hh), copied as they lie
    const rsrc_t rP = __builtin_amdgcn_make_buffer_rsrc((void*)uniform_ptr(a.P1), 0, (int)p_total, 0x00020000);
    auto issue_p = [&](int ra) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int piece = 2 * ra + (j & 1);
        const int voff = (piece < pch) ? (((t0 >> 5) + (j >> 1)) * pch + piece) * kFmChunkBytes + lt * 16 : kOobOffset;
        p_raw[j] = buf_load16(rP, voff);    // token tiles past the end of the buffer read 0
      }
    };
    auto commit_p = [&](int pb) {
#pragma unroll
      for (int j = 0; j < 4; ++j) ((u4*)ptile[pb])[j * 256 + lt] = p_raw[j];
    };

    // prologue: tile 0 and the first P1 tile into LDS, tile 1 and the second P1 tile in flight
    tile_src(c_begin, 0);
#pragma unroll
    for (int p = 0; p < 8; ++p) issue_pass(p);
    issue_p(0);
    tile_src(c_begin + (per_chunk > 1 ? 0 : 1), per_chunk > 1 ? 1 : 0);
#pragma unroll
    for (int p = 0; p < 8; ++p) { commit_pass(0, p); issue_pass(p); }
    commit_p(0);
    issue_p(1 % nA);
    __syncthreads();

    int it = 0, ac = 0;
    auto next2_src = [&](int c, int j) {                 // source of the tile two ahead of (c, j); past the end: nothing
      int c2 = c, j2 = j + 2;
      if (j2 >= per_chunk) { j2 -= per_chunk; ++c2; }
      tile_src(c2, j2);
    };
    for (int c = c_begin; c < nchunks; ++c) {
      for (int ra = 0; ra < nA; ++ra) {
        next2_src(c, ra);
#pragma unroll
        for (int p = 0; p < 8; ++p) { commit_pass((it + 1) & 1, p); issue_pass(p); }
        commit_p((ac + 1) & 1);
        issue_p((ra + 2) % nA);
        __syncthreads();
        ++it; ++ac;
      }
      for (int s = 0; s < NS; ++s) {
        next2_src(c, nA + s);
#pragma unroll
        for (int p = 0; p < 8; ++p) { commit_pass((it + 1) & 1, p); issue_pass(p); }
        __syncthreads();
        ++it;
      }
      if constexpr (NS2 > 0) {
        // sub-tiles NS .. NS+NS2-1: the MFMAs of step f run between the staging passes of the stream
#pragma unroll
        for (int s = 0; s < NS2; ++s) {
          next2_src(c, nA + NS + s);
          stage_b2(wt_lds[it & 1], z2[s], s0 + (NS + s) * kTile < s_end, [&](int f) {
            commit_pass((it + 1) & 1, f);
            issue_pass(f);
          });
          __syncthreads();
          ++it;
        }
      }
    }
    }
    if constexpr (NS2 > 0) write_z(z2, a, fsplit, fs, t0, s0 + NS * kTile, s0 + slice_w, wave, l32, g);
    return;
  }

  // =======================================================================================================
  // Compute wavefronts
  // =======================================================================================================
  f16v z[NS][2], y[2];
#pragma unroll
  for (int s = 0; s < NS; ++s) { z[s][0] = zero16(); z[s][1] = zero16(); }
  y[0] = zero16(); y[1] = zero16();
  h8 gq[8][2];

  // ---- one stage of phase A: y += V_1 tile^T (features 32*wave..) x P1^T, operands fetched from LDS one step ahead
  auto stage_a = [&](const _Float16* wb, const h8 (*pb)[64], int c, bool lastA) {
    h8 wf = tr_frag(wb + trA, wb + trA + 4 * kRow);
    h8 pf0 = pb[0][lane], pf1 = pb[8][lane];
#pragma unroll
    for (int st = 0; st < 8; ++st) {
      h8 wf_next = wf, pn0 = pf0, pn1 = pf1;
      if (st < 7) {
        const int hh = (st + 1) >> 2, kk = (st + 1) & 3;
        const _Float16* q = wb + trA + (64 * hh + 8 * kk) * kRow;
        wf_next = tr_frag(q, q + 4 * kRow);
        pn0 = pb[hh * 4 + kk][lane];
        pn1 = pb[8 + hh * 4 + kk][lane];
      }
      y[0] = mfma32(wf, pf0, y[0]);   // rows f, cols tokens
      y[1] = mfma32(wf, pf1, y[1]);
      wf = wf_next; pf0 = pn0; pf1 = pn1;
    }
    if (lastA) {
      // bias, phi, fp16, publish in operand order for phase B
      const rsrc_t rB = rsrc_at(a.b1, a.b1 ? (long long)F * 2 : 0, (long long)c * kFfnBF * 2);
      f4v bias[4];
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const u2 raw = buf_load8(rB, (32 * wave + 8 * jj + 4 * g) * 2);
        if constexpr (PK) bias[jj] = a.w_dt == DT_BF16 ? raw_to_f4<DT_BF16>(raw) : raw_to_f4<DT_F16>(raw);
        else bias[jj] = raw_to_f4<WT>(raw);
      }
      auto publish = [&](auto phi) {
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
          for (int t = 0; t < 2; ++t) {
            h8 r;
#pragma unroll
            for (int i = 0; i < 8; ++i) r[i] = (_Float16)phi(y[tt][8 * t + i] + bias[2 * t + (i >> 2)][i & 3]);
            gtile[wave][t][tt][lane] = r;
          }
      };
      if (a.act == 0) publish([](float x) { return gelu_erf_f(x); });
      else if (a.act == 1) publish([](float x) { return gelu_tanh_f(x); });
      else publish([](float x) { return fmaxf(x, 0.f); });
      y[0] = zero16(); y[1] = zero16();
    }
  };
  // ---- one sub-stage of phase B: z[s] += U_2 tile^T (ranks 128 s + 32*wave..) x Y^T
  auto stage_b = [&](const _Float16* wb, f16v (&zs)[2], bool active) {
    h8 wf = tr_frag(wb + trB, wb + trB + 8 * kRow);
#pragma unroll
    for (int fs = 0; fs < 8; ++fs) {
      h8 wf_next = wf;
      if (fs < 7) {
        const _Float16* q = wb + trB + 16 * (fs + 1) * kRow;
        wf_next = tr_frag(q, q + 8 * kRow);
      }
      if (active) {
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) zs[tt] = mfma32(wf, gq[fs][tt], zs[tt]);   // rows ranks, cols tokens
      }
      wf = wf_next;
    }
  };

  __syncthreads();   // prologue of the loader wavefronts
  int wb = 0, pb = 0;   // buffers of the weight tile / P1 tile in use
  for (int c = c_begin; c < nchunks; ++c) {
    for (int ra = 0; ra < nA; ++ra) {
      stage_a(wt_lds[wb], ptile[pb], c, ra + 1 == nA);
      __syncthreads();
      wb = nxt(wb); pb = nxt(pb);
    }
#pragma unroll
    for (int fs = 0; fs < 8; ++fs)
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) gq[fs][tt] = gtile[fs >> 1][fs & 1][tt][lane];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      stage_b(wt_lds[wb], z[s], s0 + s * kTile < s_end);
      __syncthreads();
      wb = nxt(wb);
    }
#pragma unroll
    for (int s = 0; s < NS2; ++s) {   // the loader wavefronts' sub-tiles
      __syncthreads();
      wb = nxt(wb);
    }
  }

  write_z(z, a, fsplit, fs, t0, s0, s0 + slice_w, wave, l32, g);
}

// Sum of the fp32 partial results over the splits of F -> fragment-major fp16 Z.  One thread per 16-byte FM unit
// (8 ranks of one token); the partial layout [split][rank / 4][token][4] makes the reads of a wavefront contiguous.
__global__ void __launch_bounds__(256) ffn_reduce_kernel(const float* __restrict__ part, int fsplit, int T, int r2, _Float16* Z,
                                                         size_t units) {
  const size_t u = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (u >= units) return;
  const int zch = (r2 + 63) / 64;
  const int lane = u & 63, kk = (u >> 6) & 3;
  const size_t blk = u >> 8;
  const int c = blk % zch, tile = blk / zch;
  const int tok = tile * 32 + (lane & 31), k = 64 * c + 32 * (lane >> 5) + 8 * kk;
  if (tok >= T) return;
  f4v lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
  for (int f = 0; f < fsplit; ++f) {   // fixed order: the result does not depend on scheduling
    const float* p = part + (((size_t)f * (zch * 16) + (k >> 2)) * T + tok) * 4;
    const f4v a0 = *(const f4v*)p, a1 = *(const f4v*)(p + (size_t)T * 4);
#pragma unroll
    for (int i = 0; i < 4; ++i) { lo[i] += a0[i]; hi[i] += a1[i]; }
  }
  h8 o;
#pragma unroll
  for (int i = 0; i < 4; ++i) { o[i] = (_Float16)lo[i]; o[4 + i] = (_Float16)hi[i]; }
  *(h8*)(Z + u * 8) = o;
}

template <int NS, int NS2>
hipError_t launch_ns(const FfnCoreArgs& a, const FfnCorePlan& pl, hipStream_t s) {
  const dim3 grid(((a.T + kFfnBT - 1) / kFfnBT) * pl.nslices * pl.fsplit), block(512);
  if (a.tiled) hipLaunchKernelGGL((ffn_core_kernel<NS, NS2, kWtTiled>), grid, block, 0, s, a, pl.nslices, pl.slice_w, pl.fsplit);
  else if (a.w_dt == DT_F16) hipLaunchKernelGGL((ffn_core_kernel<NS, NS2, DT_F16>), grid, block, 0, s, a, pl.nslices, pl.slice_w, pl.fsplit);
  else hipLaunchKernelGGL((ffn_core_kernel<NS, NS2, DT_BF16>), grid, block, 0, s, a, pl.nslices, pl.slice_w, pl.fsplit);
  return hipGetLastError();
}
}  // namespace

// Which kernel serves prepacked weights: the all-wavefront kernel (fsvd_ffn_wide.hip) where a workgroup has to cover
// more than 512 output ranks (there the two-role kernel parks half of its accumulators in the loader wavefronts and
// runs their MFMAs in stages of their own); measured on one machine, it is ahead from r2 = 1024 on (the decoder shape:
// 1.14 ms against 1.18 ms) and behind for r2 <= 768 (cfg2u 0.213 against 0.187 ms), where the two-role kernel stays.
// FSVD_FFN_CORE=wide / tworole overrides the choice (a tuning switch).
static bool ffn_core_use_wide(int T, int r1, int r2, int F) {
  (void)T; (void)r1; (void)F;
  const char* e = getenv("FSVD_FFN_CORE");
  if (e && e[0] == 't') return false;
  if (e && e[0] == 'w') return true;
  return r2 >= 1024;
}

// Launch shape: W sub-tiles of 128 ranks per workgroup (up to 4 on the compute wavefronts, up to 4 more on the loader
// wavefronts), the slices of r2 that follow from W, and the number of parts F is split into.  Splitting F needs fp32
// partial sums in the workspace; they may take at most T * F bytes (half of what the hidden activation itself would).
// The choice minimises (rounds of workgroups over the 256 compute units) x (weight tiles and GELU passes per workgroup).
FfnCorePlan ffn_core_plan(int T, int r1, int r2, int F, bool tiled) {
  const int tiles = (T + kFfnBT - 1) / kFfnBT;
  const size_t zpad = (size_t)((r2 + 63) / 64) * 64;
  if (tiled && ffn_core_use_wide(T, r1, r2, F)) {
    // all-wavefront kernel: groups of 256 ranks, at most four per workgroup; chunks of 256 features
    const int ngroups = (r2 + 255) / 256, nsl = (ngroups + 3) / 4, np = (ngroups + nsl - 1) / nsl;
    const int nA = (r1 + 63) / 64, nchunks = (F + 255) / 256;
    FfnCorePlan best{};
    double best_cost = 0.0;
    for (int fsplit = 1; fsplit <= nchunks; fsplit *= 2) {
      const size_t part = fsplit > 1 ? (size_t)fsplit * zpad * T * 4 : 0;
      if (part > (size_t)T * F) break;
      const long wgs = (long)tiles * nsl * fsplit;
      const double rounds = (double)((wgs + 255) / 256);
      const double cost = rounds * ((nchunks + fsplit - 1) / fsplit) * (nA + 4.0 * np + 3.0) + 4.0 * (fsplit > 1);
      if (best.nslices == 0 || cost < best_cost - 1e-9) {
        best_cost = cost;
        best.nslices = nsl; best.slice_w = 256 * np; best.ns = 0; best.ns2 = 0; best.fsplit = fsplit; best.wide = np;
        best.partial_bytes = part;
      }
    }
    return best;
  }
  const int nsub = (r2 + kTile - 1) / kTile, nA = (r1 + kTile - 1) / kTile, nchunks = (F + kFfnBF - 1) / kFfnBF;
  FfnCorePlan best{};
  double best_cost = 0.0;
  for (int W = 1; W <= 8; ++W) {
    const int nsl = (nsub + W - 1) / W;
    int slice_w = (r2 + nsl - 1) / nsl;
    slice_w = (slice_w + kTile - 1) / kTile * kTile;   // whole sub-tiles (tile images are addressed by tile)
    const int w_eff = (slice_w + kTile - 1) / kTile;
    if (w_eff != W) continue;                               // the same shape is reached with a smaller W
    for (int fsplit = 1; fsplit <= nchunks; fsplit *= 2) {
      const size_t part = fsplit > 1 ? (size_t)fsplit * zpad * T * 4 : 0;
      if (part > (size_t)T * F) break;
      const long wgs = (long)tiles * nsl * fsplit;
      const double rounds = (double)((wgs + 255) / 256);
      const int on_loader = W > 4 ? W - 4 : 0;
      const double per_chunk = 1.2 * nA + (W - on_loader) + 1.25 * on_loader + 1.5;
      const double cost = rounds * ((nchunks + fsplit - 1) / fsplit) * per_chunk + 2.0 * (fsplit > 1);
      if (best.nslices == 0 || cost < best_cost - 1e-9) {
        best_cost = cost;
        best.nslices = nsl; best.slice_w = slice_w; best.ns = W - on_loader; best.ns2 = on_loader; best.fsplit = fsplit;
        best.wide = 0;
        best.partial_bytes = part;
      }
    }
  }
  return best;
}

hipError_t launch_ffn_core(const FfnCoreArgs& a, hipStream_t s) {
  const FfnCorePlan pl = ffn_core_plan(a.T, a.r1, a.r2, a.F, a.tiled != 0);
  if (pl.fsplit > 1 && !a.Zpart) return hipErrorInvalidValue;
  hipError_t e = hipErrorInvalidValue;
  if (pl.wide > 0) e = launch_ffn_core_wide(a, pl, s);
  else switch (pl.ns * 8 + pl.ns2) {
    case 1 * 8 + 0: e = launch_ns<1, 0>(a, pl, s); break;
    case 2 * 8 + 0: e = launch_ns<2, 0>(a, pl, s); break;
    case 3 * 8 + 0: e = launch_ns<3, 0>(a, pl, s); break;
    case 4 * 8 + 0: e = launch_ns<4, 0>(a, pl, s); break;
    case 4 * 8 + 1: e = launch_ns<4, 1>(a, pl, s); break;
    case 4 * 8 + 2: e = launch_ns<4, 2>(a, pl, s); break;
    case 4 * 8 + 3: e = launch_ns<4, 3>(a, pl, s); break;
    case 4 * 8 + 4: e = launch_ns<4, 4>(a, pl, s); break;
  }
  if (e != hipSuccess || pl.fsplit == 1) return e;
  const size_t units = fm_bytes(a.T, a.r2) / 16;
  hipLaunchKernelGGL(ffn_reduce_kernel, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, s, a.Zpart, pl.fsplit, a.T, a.r2,
                     (_Float16*)a.Z, units);
  return hipGetLastError();
}

}  // namespace fsvd
