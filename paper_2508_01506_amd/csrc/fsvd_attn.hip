// Streaming attention over rank-space inputs (Alg. 1): Q, K and V tiles are rebuilt on chip from
// P_q, P_k, P_v [T, r] (fragment-major fp16) and the head's columns of V_q, V_k, V_v [r, D] (Alg. 1 Part I),
// scores and the streaming softmax never leave registers (Part II), and only the context C [T, D] is
// written (fragment-major fp16).
//
// One workgroup (8 wavefronts, two per SIMD so that one wavefront's softmax / waits overlap the other's
// MFMAs) owns one (sequence, head, block of BQ = 256*QT queries).
//   Q phase : every wavefront rebuilds Q^T [d_h, 32*QT] for its own queries, contraction over r_q
//             in 64-wide chunks, pre-scaled by softmax_scale*log2(e), and keeps it as MFMA operands.
//   KV loop : per step of BKV keys (128 for d_h = 128, 256 for long sequences with d_h = 64) the wavefronts
//             rebuild the K and V tiles: half of them K, half V, each a tile of KTW x DTW 32x32 blocks of
//             (V_a[:, head])^T P_a^T (features x keys) - one loop without role-dependent code.  Weight chunks
//             [64 ranks, d_h] are copied into LDS (double-buffered, staging passes spread between the MFMA
//             steps), shared, and read back transposed through a rolling window; P operands come straight from
//             global memory (fragment-major).  K^T is published in LDS in operand order, V as rows [key][d]
//             that the context product reads back with the transposing read.  Then every wavefront computes
//             S^T = K Q^T for its queries, masks, updates the (lazily raised) row maximum and the row sum and
//             accumulates O^T += V^T P~^T.
// All products are arranged "transposed" (keys or features along accumulator rows, queries along
// lanes), so the accumulators of one product are, after rounding to fp16, exactly the operand
// registers of the next one: no activation ever needs a transpose or an LDS round trip except the
// K/V tile exchange between wavefronts, and the softmax row statistics are per-lane scalars.
#include "fsvd_common.h"
#include "fsvd_kernels.h"

#include <stdlib.h>

namespace fsvd {

namespace {

constexpr int kAttnWaves = 8;
constexpr int kAttnThreads = kAttnWaves * 64;
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ h8 pack8(const f16v& x, int t, float add) {
  h8 r;
#pragma unroll
  for (int i = 0; i < 8; ++i) r[i] = (_Float16)(x[8 * t + i] + add);
  return r;
}
__device__ __forceinline__ h8 pack8(const f16v& x, int t) {   // no "+ 0.f": that is not a no-op and would cost an add per element
  h8 r;
#pragma unroll
  for (int i = 0; i < 8; ++i) r[i] = (_Float16)x[8 * t + i];
  return r;
}

template <int DH, int QT, int WT>
__global__ void __launch_bounds__(kAttnThreads, 1) attn_core_kernel(AttnCoreArgs a, int nqb) {
  constexpr int DT32 = DH / 32;             // 32-wide feature tiles
  constexpr int DST = DH / 16;              // 16-wide contraction steps over d_h
  constexpr int BQ = kAttnWaves * QT * 32;  // queries per workgroup
  // K/V rebuild: wavefront tile = KTW key tiles x DTW feature tiles of one matrix (operands reused KTW resp. DTW times);
  // 2 matrices x (NKT / KTW) key groups x (DT32 / DTW) feature groups = 8 wavefronts
  constexpr int KTW = (DH == 64 && QT == 1) ? 1 : (DH == 128 ? 1 : 2);
  constexpr int DTW = DH == 128 ? 4 : 2;    // d_h = 128: all four feature tiles, so that no two wavefronts load the same P operands
  constexpr int NDG = DT32 / DTW;           // feature groups
  constexpr int NKT = (kAttnWaves / 2 / NDG) * KTW;   // 32-key tiles per step
  constexpr int BKV = 32 * NKT;             // keys per step
  constexpr int WS = wtile_stride(DH);      // halves per LDS row of a staged weight chunk [64 ranks][DH]
  constexpr int WBUF = kChunkK * WS;        // halves per staged weight chunk (one matrix)
  constexpr int LPR = DH / 8;               // lanes per chunk row while staging (16 bytes each)
  constexpr int RPP = kAttnThreads / LPR;   // chunk rows staged per pass
  constexpr int NP = kChunkK / RPP;         // passes (loads per thread) per matrix chunk

  __shared__ __attribute__((aligned(16))) _Float16 wbuf[2][2][WBUF];   // [parity][K|V weights]
  __shared__ __attribute__((aligned(16))) h8 ktile[NKT][DST][64];
  __shared__ __attribute__((aligned(16))) _Float16 vtile[BKV * WS];   // V [key][d] row-major, read back transposed

  const int tid = threadIdx.x;
  const int lane = tid & 63, l32 = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps everything derived from it scalar
  const int BH = a.B * a.H;
  const int bh = blockIdx.x % BH;
  const int qb = nqb - 1 - blockIdx.x / BH;   // late query blocks (most keys under a causal mask) first
  const int b = bh / a.H, h = bh % a.H;
  const int M = a.M, D = a.D, T = a.B * a.M;
  const int q0 = qb * BQ;
  const int qw = q0 + wave * QT * 32;         // first query of this wavefront
  int kv_len = a.key_len ? a.key_len[b] : M;
  kv_len = kv_len < 1 ? 1 : (kv_len > M ? M : kv_len);
  int kv_end = kv_len;
  if (a.causal && q0 + BQ < kv_end) kv_end = q0 + BQ;
  const int nsteps = (kv_end + BKV - 1) / BKV;
  const int tok0 = b * M;
  const int col0 = h * DH;                    // this head's columns in V_a, b_a and C

  // ---- weight staging: thread -> chunk row s_r (+ RPP per pass), 8 head columns from s_c
  const int s_r = tid / LPR, s_c = 8 * (tid % LPR);
  const int trA = tr_lane_off(lane, WS) + 32 * g * WS;   // transposing-read base of this lane (halves)
  const int trV = tr_lane_off(lane, WS) + 4 * g * WS;    // same for the V tile: keys 16 t + 4 g + {0..3, 8..11}
  // Prepacked weights (tile images, whole-matrix factors only): byte offset of the 8 columns this thread stages of rank
  // row rho.  The column part is fixed per thread (chunks start at multiples of 64 rows, so rho % 4 == s_r % 4).
  constexpr int ST = WT == kWtTiled ? DT_F16 : WT;          // type of the values as they arrive for staging
  const int tl_ntn = (D + 127) / 128;
  const int tl_n = (col0 + s_c) & 127;
  const int tl_col = ((col0 + s_c) >> 7) * kTileImageBytes + ((((tl_n >> 5) ^ (s_r & 3)) << 5) + (tl_n & 31)) * 2;
  auto tiled_off = [&](int rho) { return (rho >> 7) * tl_ntn * kTileImageBytes + (rho & 127) * 256 + tl_col; };
  // 4 consecutive bias entries of this head, as floats
  auto bias4 = [&](const void* bp, int d) -> f4v {
    const rsrc_t r = rsrc_at(bp, bp ? (long long)D * 2 : 0, 0);
    const u2 raw = buf_load8(r, (col0 + d) * 2);
    if constexpr (WT == kWtTiled) return a.w_dt == DT_BF16 ? raw_to_f4<DT_BF16>(raw) : raw_to_f4<DT_F16>(raw);
    else return raw_to_f4<WT>(raw);
  };

  // =================================== Q phase ===================================
  h8 qf[DST][QT];
  {
    f16v acc[DT32][QT];
#pragma unroll
    for (int dt = 0; dt < DT32; ++dt)
#pragma unroll
      for (int qt = 0; qt < QT; ++qt) acc[dt][qt] = zero16();
    // rank window of this head in V_q / P_q: all of [0, r_q) for whole-matrix factors, [h r_q, (h+1) r_q) of the
    // concatenated ranks for per-head factors; chunks are 64 ranks of the concatenated axis
    const int lo = a.per_head ? (h / a.per_head) * a.rq : 0, hi = lo + a.rq;
    const int c0 = lo / kChunkK, nc = (hi - 1) / kChunkK - c0 + 1;
    const int ld = a.per_head ? a.per_head * DH : D, wcol0 = a.per_head ? (h % a.per_head) * DH : col0;
    const int rtot = a.per_head ? (a.H / a.per_head) * a.rq : a.rq;
    const int pchq = (rtot + kChunkK - 1) / kChunkK;
    const long long p_total = (long long)fm_bytes(T, rtot);
    const long long w_total = (long long)rtot * ld * 2;
    int voffP[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
      int q = qw + 32 * qt + l32;
      q = q < M ? q : M - 1;
      voffP[qt] = fm_voff(tok0 + q, pchq, g);
    }
    u4 w_raw[NP];
    h8 pfr[QT][4];
    auto load_p = [&](int c, int kk) {   // the rank padding of an FM tensor holds zeros: no tail handling
      const rsrc_t r = rsrc_at(a.Pq, p_total, (long long)(c0 + c) * kFmChunkBytes);
#pragma unroll
      for (int qt = 0; qt < QT; ++qt) pfr[qt][kk] = __builtin_bit_cast(h8, buf_load16(r, voffP[qt] + kk * kFmStepBytes));
    };
    auto issue_w = [&](int c) {
      const rsrc_t r = WT == kWtTiled ? rsrc_at(a.Vq, (long long)tiled_bytes(rtot, D), 0)
                                      : rsrc_at(a.Vq, w_total, ((long long)(c0 + c) * kChunkK * ld + wcol0) * 2);
#pragma unroll
      for (int p = 0; p < NP; ++p) {
        const int rho = (c0 + c) * kChunkK + s_r + p * RPP;          // ranks outside the window contribute nothing
        const int off = WT == kWtTiled ? tiled_off(rho) : ((s_r + p * RPP) * ld + s_c) * 2;
        w_raw[p] = buf_load16(r, (rho >= lo && rho < hi) ? off : kOobOffset);
      }
    };
    auto commit_w = [&](int pb) {
#pragma unroll
      for (int p = 0; p < NP; ++p) stage_store16<ST>(&wbuf[pb][0][(s_r + p * RPP) * WS + s_c], w_raw[p]);
    };
    issue_w(0);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) load_p(0, kk);
    commit_w(0);
    if (nc > 1) issue_w(1);
    __syncthreads();
    for (int c = 0; c < nc; ++c) {
      const bool more = c + 1 < nc;
      if (more) commit_w((c + 1) & 1);       // chunk c+1 arrived during the previous iteration
      if (c + 2 < nc) issue_w(c + 2);        // chunk c+2 has this whole iteration to land
      const _Float16* wb = wbuf[c & 1][0];
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        h8 wf[DT32];
#pragma unroll
        for (int dt = 0; dt < DT32; ++dt) {
          const _Float16* q = wb + trA + 8 * kk * WS + 32 * dt;
          wf[dt] = tr_frag(q, q + 4 * WS);
        }
#pragma unroll
        for (int dt = 0; dt < DT32; ++dt)
#pragma unroll
          for (int qt = 0; qt < QT; ++qt) acc[dt][qt] = mfma32(wf[dt], pfr[qt][kk], acc[dt][qt]);
        if (more) load_p(c + 1, kk);     // refill the operand registers just consumed
      }
      __syncthreads();
    }
    // bias, softmax scale (log2 domain), round to fp16 operands
    const float qs = a.scale * kLog2e;
#pragma unroll
    for (int dt = 0; dt < DT32; ++dt) {
      f4v bias[4];
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) bias[jj] = bias4(a.bq, 32 * dt + 8 * jj + 4 * g);
#pragma unroll
      for (int qt = 0; qt < QT; ++qt)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          h8 r;
#pragma unroll
          for (int i = 0; i < 8; ++i) r[i] = (_Float16)((acc[dt][qt][8 * t + i] + bias[2 * t + (i >> 2)][i & 3]) * qs);
          qf[2 * dt + t][qt] = r;
        }
    }
  }

  // =================================== KV loop ===================================
  f16v o[DT32][QT];
  // Softmax state per query (lane): reference maximum and row sum.
  float m_run[QT], l_run[QT];
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    m_run[qt] = 0.f;
    l_run[qt] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT32; ++dt) o[dt][qt] = zero16();
  }
  bool first = true;       // no key block has been folded in yet (wave-uniform)

  const int which = wave & 1;                 // 0: keys, 1: values
  const int kt0 = ((wave >> 1) / NDG) * KTW;  // first key tile of this wavefront
  const int dt0 = ((wave >> 1) % NDG) * DTW;  // first feature tile of this wavefront
  const char* const Psrc = which ? uniform_ptr(a.Pv) : uniform_ptr(a.Pk);
  const char* const bsel = which ? uniform_ptr(a.bv) : uniform_ptr(a.bk);
  // rank windows of this head in (V_k, P_k) and (V_v, P_v), as in the Q phase
  const int lo_k = a.per_head ? (h / a.per_head) * a.rk : 0, hi_k = lo_k + a.rk;
  const int lo_v = a.per_head ? (h / a.per_head) * a.rv : 0, hi_v = lo_v + a.rv;
  const int c0_k = lo_k / kChunkK, nch_k = (hi_k - 1) / kChunkK - c0_k + 1;
  const int c0_v = lo_v / kChunkK, nch_v = (hi_v - 1) / kChunkK - c0_v + 1;
  const int ld = a.per_head ? a.per_head * DH : D, wcol0 = a.per_head ? (h % a.per_head) * DH : col0;
  const int rtot_k = a.per_head ? (a.H / a.per_head) * a.rk : a.rk, rtot_v = a.per_head ? (a.H / a.per_head) * a.rv : a.rv;
  const long long wt_k = (long long)rtot_k * ld * 2, wt_v = (long long)rtot_v * ld * 2;
  // the P operands of this wavefront's role
  const int rtot_p = which ? rtot_v : rtot_k;
  const int pch = (rtot_p + kChunkK - 1) / kChunkK;
  const int c0_p = which ? c0_v : c0_k, nch_p = which ? nch_v : nch_k;
  const long long p_total = (long long)fm_bytes(T, rtot_p);
  const int nc = nch_k > nch_v ? nch_k : nch_v;
  const int total = nsteps * nc;
  // per-lane staging offsets of the two weight matrices for relative chunk c (rows outside the window: nothing)
  auto w_voff = [&](int m, int c, int pp) {
    const int rho = ((m ? c0_v : c0_k) + c) * kChunkK + s_r + pp * RPP;
    const bool ok = m ? (rho >= lo_v && rho < hi_v) : (rho >= lo_k && rho < hi_k);
    const int off = WT == kWtTiled ? tiled_off(rho) : ((s_r + pp * RPP) * ld + s_c) * 2;
    return ok ? off : kOobOffset;
  };
  const long long ti_k = (long long)tiled_bytes(rtot_k, D), ti_v = (long long)tiled_bytes(rtot_v, D);
  auto w_rsrc = [&](int m, int c, bool live) {
    if constexpr (WT == kWtTiled) return rsrc_at(m ? a.Vv : a.Vk, live ? (m ? ti_v : ti_k) : 0, 0);
    else return rsrc_at(m ? a.Vv : a.Vk, live ? (m ? wt_v : wt_k) : 0, ((long long)((m ? c0_v : c0_k) + c) * kChunkK * ld + wcol0) * 2);
  };

  u4 w_raw[2][NP];
  auto issue_w = [&](int c) {
#pragma unroll
    for (int m = 0; m < 2; ++m) {
      const rsrc_t r = w_rsrc(m, c, true);
#pragma unroll
      for (int p = 0; p < NP; ++p) w_raw[m][p] = buf_load16(r, w_voff(m, c, p));
    }
  };
  auto commit_w = [&](int pb) {
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
      for (int p = 0; p < NP; ++p) stage_store16<ST>(&wbuf[pb][m][(s_r + p * RPP) * WS + s_c], w_raw[m][p]);
  };
  h8 pfr[KTW][4];
  int voffKV[KTW];
  auto set_keys = [&](int step) {
#pragma unroll
    for (int i = 0; i < KTW; ++i) {
      int key = step * BKV + 32 * (kt0 + i) + l32;
      key = key < M ? key : M - 1;
      voffKV[i] = fm_voff(tok0 + key, pch, g);
    }
  };
  auto load_p = [&](int c, int kk) {      // chunks past this matrix's rank fall outside the resource: 0
    const rsrc_t r = rsrc_at(Psrc, (c < nch_p) ? p_total : 0, (long long)(c0_p + c) * kFmChunkBytes);
#pragma unroll
    for (int i = 0; i < KTW; ++i) pfr[i][kk] = __builtin_bit_cast(h8, buf_load16(r, voffKV[i] + kk * kFmStepBytes));
  };

  f16v acc[KTW][DTW];
#pragma unroll
  for (int i = 0; i < KTW; ++i)
#pragma unroll
    for (int j = 0; j < DTW; ++j) acc[i][j] = zero16();

  if (total > 0) {
    issue_w(0);
    set_keys(0);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) load_p(0, kk);
    commit_w(0);
    if (total > 1) issue_w(nc > 1 ? 1 : 0);
  }
  __syncthreads();

  int step = 0, c = 0;
  for (int it = 0; it < total; ++it) {
    const bool more = it + 1 < total;
    int nstep = step, ncn = c + 1;
    if (ncn == nc) { ncn = 0; nstep = step + 1; }
    if (ncn == 0) set_keys(nstep);                       // the refills below already belong to the next step
    {
      // Chunk it+1 (requested during the previous iteration) is converted and written to the other LDS buffer and
      // chunk it+2 is requested, one staging pass per MFMA step, so that the LDS writes and the global requests of
      // the eight wavefronts spread over the iteration instead of bursting after the barrier.  Past the last chunk
      // the resources have size 0: the loads return zeros and nothing branches.
      const int c2 = ncn + 1 == nc ? 0 : ncn + 1;
      const rsrc_t rw0 = w_rsrc(0, c2, it + 2 < total);
      const rsrc_t rw1 = w_rsrc(1, c2, it + 2 < total);
      const rsrc_t rp = rsrc_at(Psrc, (more && ncn < nch_p) ? p_total : 0, (long long)(c0_p + ncn) * kFmChunkBytes);
      _Float16* const wnext = wbuf[(it + 1) & 1][0];
      // both roles compute (weights^T) x (P^T): rows = features, columns = keys, so the loop has no role-dependent code
      const _Float16* wb = wbuf[it & 1][which] + trA + 32 * dt0;
      // The 4 DTW weight fragments of the chunk pass through a rolling window of kWin registers sets: fragment
      // f + kWin is requested from LDS right after fragment f has been consumed, kWin MFMA groups ahead of its use.
      constexpr int NF = 4 * DTW, kWin = 4;
      auto read_w = [&](int f) {
        const _Float16* q = wb + 8 * (f / DTW) * WS + 32 * (f % DTW);
        return tr_frag(q, q + 4 * WS);
      };
      h8 win[kWin];
#pragma unroll
      for (int f = 0; f < kWin; ++f) win[f] = read_w(f);
#pragma unroll
      for (int f = 0; f < NF; ++f) {
        const int kk = f / DTW, j = f % DTW;
#pragma unroll
        for (int i = 0; i < KTW; ++i) acc[i][j] = mfma32(win[f % kWin], pfr[i][kk], acc[i][j]);   // rows d, cols keys
        if (f + kWin < NF) win[f % kWin] = read_w(f + kWin);
        if (j == DTW - 1) {
          // refill the operand registers just consumed
#pragma unroll
          for (int i = 0; i < KTW; ++i) pfr[i][kk] = __builtin_bit_cast(h8, buf_load16(rp, voffKV[i] + kk * kFmStepBytes));
          if ((kk * 2 * NP) % 4 == 0) {   // staging pass q of 2 NP, spread evenly over the four steps
            constexpr int kPassesPerStep = (2 * NP + 3) / 4;
#pragma unroll
            for (int u = 0; u < kPassesPerStep; ++u) {
              const int q = kk * 2 * NP / 4 + u;
              const int m = q / NP, pp = q % NP;
              stage_store16<ST>(wnext + m * WBUF + (s_r + pp * RPP) * WS + s_c, w_raw[m][pp]);
              w_raw[m][pp] = buf_load16(m ? rw1 : rw0, w_voff(m, c2, pp));
            }
          }
        }
        __builtin_amdgcn_sched_barrier(0);   // keep the window rolling in this order
      }
    }
    __syncthreads();

    if (c == nc - 1) {
      // ---- publish the rebuilt tiles (bias added, fp16): K^T in operand order; V as rows of [key][d], which the
      // transposing LDS read turns into the V^T operand of the context product
#pragma unroll
      for (int j = 0; j < DTW; ++j) {
        f4v bias[4];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) bias[jj] = bias4(bsel, 32 * (dt0 + j) + 8 * jj + 4 * g);
#pragma unroll
        for (int i = 0; i < KTW; ++i) {
          if (which == 0) {
#pragma unroll
            for (int t = 0; t < 2; ++t) {
              h8 r;
#pragma unroll
              for (int e = 0; e < 8; ++e) r[e] = (_Float16)(acc[i][j][8 * t + e] + bias[2 * t + (e >> 2)][e & 3]);
              ktile[kt0 + i][2 * (dt0 + j) + t][lane] = r;
            }
          } else {
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
              h4 r;
#pragma unroll
              for (int e = 0; e < 4; ++e) r[e] = (_Float16)(acc[i][j][4 * jj + e] + bias[jj][e]);
              *(h4*)&vtile[(32 * (kt0 + i) + l32) * WS + 32 * (dt0 + j) + 8 * jj + 4 * g] = r;
            }
          }
        }
      }
      __syncthreads();

      // ---- scores, streaming softmax, context for this wavefront's queries
      const int qlast = qw + 32 * QT - 1;
      // The reference maximum is subtracted by the matrix core: one more contraction step whose K-side operand is 1 in
      // two slots and whose Q-side operand holds -m_run of the lane's query, split into an fp16 head and tail (together
      // they carry m_run to about 2^-22 relative).  The scores then leave the accumulators as S - m_run at the price of
      // one MFMA per score tile instead of 16 vector subtractions.
      h8 kone = {}, qneg[QT];
      kone[0] = g == 0 ? (_Float16)1.0f : (_Float16)0.0f;
      kone[1] = kone[0];
      auto set_qneg = [&](int qt) {
        const _Float16 hi = (_Float16)(-m_run[qt]);
        const _Float16 lo = (_Float16)(-m_run[qt] - (float)hi);
        qneg[qt] = h8{};
        qneg[qt][0] = g == 0 ? hi : (_Float16)0.0f;
        qneg[qt][1] = g == 0 ? lo : (_Float16)0.0f;
      };
#pragma unroll
      for (int qt = 0; qt < QT; ++qt) set_qneg(qt);
#pragma unroll 1
      for (int ks = 0; ks < NKT; ++ks) {
        const int key0 = step * BKV + 32 * ks;
        if (key0 >= kv_end) break;
        if (a.causal && key0 > qlast) break;
        f16v s[QT];
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) s[qt] = mfma32(kone, qneg[qt], zero16());   // -m_run in every row of the query's column
#pragma unroll
        for (int ds = 0; ds < DST; ++ds) {
          const h8 kf = ktile[ks][ds][lane];
#pragma unroll
          for (int qt = 0; qt < QT; ++qt) s[qt] = mfma32(kf, qf[ds][qt], s[qt]);   // S^T - m: rows keys, cols queries
        }
        const bool need_mask = (key0 + 32 > kv_len) || (a.causal && key0 + 31 > qw);
        if (need_mask) {
#pragma unroll
          for (int qt = 0; qt < QT; ++qt) {
            const int q = qw + 32 * qt + l32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const int key = key0 + 8 * (v >> 2) + 4 * g + (v & 3);
              if (key >= kv_len || (a.causal && key > q)) s[qt][v] = -INFINITY;
            }
          }
        }
        // Lazy running maximum (log2 domain): the reference maximum of a row is raised, and O and l rescaled, only when
        // the slab's maximum exceeds it by more than 8; until then the probabilities are at most 2^8, which fp16
        // holds with full relative precision.  The softmax does not depend on the reference, so nothing changes
        // but the number of rescalings (one per row for most inputs instead of one per slab).  s already is S - m_run.
        // The first slab sets the reference to its own maximum (key 0 is visible to every query, so it is finite).
        h8 pf[QT][2];
        float mx[QT];
        bool raise = first;
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
          float m = s[qt][0];
#pragma unroll
          for (int v = 1; v < 16; ++v) m = fmaxf(m, s[qt][v]);
          mx[qt] = halves_max(m);
          raise = raise || (mx[qt] > 8.0f);
        }
        if (__any(raise)) {
#pragma unroll
          for (int qt = 0; qt < QT; ++qt) {
            // first slab: move the reference to the slab's maximum wherever it is (O and l are still zero);
            // later: only upwards
            const float delta = first ? fmaxf(mx[qt], -1e30f) : fmaxf(mx[qt], 0.f);
            const float alpha = first ? 0.f : __builtin_amdgcn_exp2f(-delta);
            m_run[qt] += delta;
            l_run[qt] *= alpha;
            set_qneg(qt);
#pragma unroll
            for (int v = 0; v < 16; ++v) s[qt][v] -= delta;
#pragma unroll
            for (int dt = 0; dt < DT32; ++dt)
#pragma unroll
              for (int v = 0; v < 16; ++v) o[dt][qt][v] *= alpha;
          }
        }
        first = false;
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
          float sum = 0.f;
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const float p = __builtin_amdgcn_exp2f(s[qt][v]);
            s[qt][v] = p;
            sum += p;
          }
          l_run[qt] += sum;
          pf[qt][0] = pack8(s[qt], 0);
          pf[qt][1] = pack8(s[qt], 1);
        }
#pragma unroll
        for (int dt = 0; dt < DT32; ++dt)
#pragma unroll
          for (int t = 0; t < 2; ++t) {
            const _Float16* vq = vtile + (32 * ks + 16 * t) * WS + trV + 32 * dt;
            const h8 vf = tr_frag(vq, vq + 8 * WS);
#pragma unroll
            for (int qt = 0; qt < QT; ++qt) o[dt][qt] = mfma32(vf, pf[qt][t], o[dt][qt]);   // O^T: rows d, cols queries
          }
      }
      // the rebuild accumulators are cleared only now, so that their registers are free during the softmax above
#pragma unroll
      for (int i = 0; i < KTW; ++i)
#pragma unroll
        for (int j = 0; j < DTW; ++j) acc[i][j] = zero16();
    }
    step = nstep;
    c = ncn;
  }

  // ---- normalise and write the context, fragment-major: 4 consecutive features per 8-byte store
  {
    _Float16* C = (_Float16*)a.C;
    const int cch = D / 64;
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
      const int q = qw + 32 * qt + l32;
      const float l = halves_sum(l_run[qt]);
      const float inv = l > 0.f ? 1.0f / l : 0.f;
      if (q < M) {
        const int tok = tok0 + q;
#pragma unroll
        for (int dt = 0; dt < DT32; ++dt) {
          const int dabs = col0 + 32 * dt;
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) {
            const size_t unit = ((size_t)((tok >> 5) * cch + (dabs >> 6)) * 4 + jj) * 64 + ((dabs >> 5) & 1) * 32 + (tok & 31);
            h4 r;
#pragma unroll
            for (int i = 0; i < 4; ++i) r[i] = (_Float16)(o[dt][qt][4 * jj + i] * inv);
            *(h4*)(C + unit * 8 + 4 * g) = r;
          }
        }
      }
    }
  }
}

template <int DH, int QT>
hipError_t launch_qt(const AttnCoreArgs& a, hipStream_t s) {
  constexpr int BQ = kAttnWaves * QT * 32;
  const int nqb = (a.M + BQ - 1) / BQ;
  const dim3 grid(a.B * a.H * nqb), block(kAttnThreads);
  if (a.tiled) hipLaunchKernelGGL((attn_core_kernel<DH, QT, kWtTiled>), grid, block, 0, s, a, nqb);
  else if (a.w_dt == DT_F16) hipLaunchKernelGGL((attn_core_kernel<DH, QT, DT_F16>), grid, block, 0, s, a, nqb);
  else hipLaunchKernelGGL((attn_core_kernel<DH, QT, DT_BF16>), grid, block, 0, s, a, nqb);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_core(const AttnCoreArgs& a, hipStream_t s) {
  const int dh = a.D / a.H;
  // one factor pair per head with k / v ranks <= 64 <= d_h: the absorbed schedule, which rebuilds no K or V tile at all
  // (FSVD_ATTN_ABSORBED=0 keeps the rebuilding kernel: a switch for comparisons)
  if (attn_absorbed_supported(a)) {
    const char* e = getenv("FSVD_ATTN_ABSORBED");
    if (!(e && e[0] == '0')) return launch_attn_absorbed(a, s);
  }
  if (dh == 64) return a.M <= 256 ? launch_qt<64, 1>(a, s) : launch_qt<64, 2>(a, s);
  if (dh == 128) return launch_qt<128, 1>(a, s);
  return hipErrorInvalidValue;
}

}  // namespace fsvd
