// C[T, N] = A[T, K] W[K, N] (+ bias) (+ residual): the rank projections P_a = X U_a, the factored
// output projection (C U_o) V_o + b_o and the two GEMMs that bracket the fused FFN kernel
// (Alg. 2 "GEMM 1st" / "GEMM 2nd").
//
// One workgroup = 4 wavefronts stacked along the rows: a 256 x BN output tile, each wavefront a
// 64 x BN slab held as 32x32 MFMA accumulators.  Activation operands go from global memory straight
// into registers (no other wavefront needs them); in the fragment-major layout that is one
// contiguous 1 KiB load per operand.  Weight tiles are copied row by row into a double-buffered LDS
// tile and read back with the LDS's transposing read by all four wavefronts: 0.5 KiB per MFMA.
// A fragment-major output is produced with the operand roles swapped (rows = output columns,
// lanes = tokens), so that each lane owns 4 consecutive output columns of one token and a wavefront
// writes contiguous 512-byte runs of the destination layout.
#include "fsvd_common.h"
#include "fsvd_kernels.h"

namespace fsvd {

namespace {

enum : int { AM_ROW_F16 = 0, AM_ROW_BF16 = 1, AM_ROW_F32 = 2, AM_FM = 3 };

template <int AM> struct RawAct { u4 v; };
template <> struct RawAct<AM_ROW_F32> { u4 lo, hi; };

template <int AM>
__device__ __forceinline__ h8 cvt_raw_act(const RawAct<AM>& r) {
  if constexpr (AM == AM_ROW_F32) {
    f4v lo = __builtin_bit_cast(f4v, r.lo), hi = __builtin_bit_cast(f4v, r.hi);
    h8 o;
    o[0] = (_Float16)lo[0]; o[1] = (_Float16)lo[1]; o[2] = (_Float16)lo[2]; o[3] = (_Float16)lo[3];
    o[4] = (_Float16)hi[0]; o[5] = (_Float16)hi[1]; o[6] = (_Float16)hi[2]; o[7] = (_Float16)hi[3];
    return o;
  } else if constexpr (AM == AM_ROW_BF16) {
    return raw_to_h8<DT_BF16>(r.v);
  } else {
    return __builtin_bit_cast(h8, r.v);
  }
}

template <int AM, int WT, int BN, bool CFM>
__global__ void __launch_bounds__(256, (AM == AM_ROW_F32) ? 1 : 2) linear_kernel(LinearArgs a, int tiles_m, int tiles_n, int ksplit) {
  constexpr int NT = BN / 32;            // 32-column MFMA tiles per wavefront
  constexpr int ESZ = (AM == AM_ROW_F32) ? 4 : 2;
  constexpr int WS = wtile_stride(BN);   // halves per LDS tile row
  constexpr int LPR = BN / 8;            // lanes per tile row while staging (16 bytes each)
  constexpr int RPP = 256 / LPR;         // tile rows staged per pass
  constexpr int NP = kChunkK / RPP;      // passes (loads per thread) per chunk
  __shared__ __attribute__((aligned(16))) _Float16 lds[2][kChunkK * WS];

  // Few rows and a long contraction (the projections of a decoding step): the contraction is split over `ksplit`
  // workgroups per tile, which write fp32 partial sums that a second kernel adds in a fixed order.
  const int ntile = tiles_m * tiles_n;
  const int ks = blockIdx.x / ntile;
  const int tile = xcd_tile(blockIdx.x % ntile, ntile);
  const int tm = tile / tiles_n;
  int tn = tile % tiles_n;
  int gi = 0, goff = 0;                 // goff: first column of this group in the concatenation of all groups' outputs
  for (; gi < a.ngroups - 1; ++gi) {
    int t = (a.g[gi].N + BN - 1) / BN;
    if (tn < t) break;
    tn -= t;
    goff += a.g[gi].N;
  }
  const LinearGroup G = a.g[gi];
  const int n0 = tn * BN;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform
  const int l32 = lane & 31, g = lane >> 5;
  const int m0 = tm * 256 + wave * 64;
  const int K = a.K, T = a.T;
  const int kchunks = (K + kChunkK - 1) / kChunkK;
  const int cps = (kchunks + ksplit - 1) / ksplit;
  const int cb = ks * cps, ce = (cb + cps < kchunks) ? cb + cps : kchunks;   // this workgroup's chunks of the contraction

  // ---- activation addressing: one 32-bit offset per 32-row tile
  const long long a_total = (AM == AM_FM) ? (long long)fm_bytes(T, K) : (long long)T * a.lda * ESZ;
  int voffA[2];
#pragma unroll
  for (int mt = 0; mt < 2; ++mt) {
    int r = m0 + 32 * mt + l32;
    if constexpr (AM == AM_FM) {
      voffA[mt] = fm_voff(r, kchunks, g);                 // rows past the last tile fall outside the resource
    } else {
      r = r < T ? r : T - 1;                              // clamped; their results are never stored
      voffA[mt] = (r * a.lda + 32 * g) * ESZ;
    }
  }
  // ---- weight staging: thread -> row s_r (+ RPP per pass), 8 columns from s_c
  const int s_r = threadIdx.x / LPR, s_c = 8 * (threadIdx.x % LPR);
  const long long w_total = WT == kWtTiled ? (long long)tiled_bytes(K, G.N) : (long long)K * G.ldw * 2;
  const bool s_ok = n0 + s_c < G.N;
  // prepacked weights (tile images): the column part of this thread's byte offset is fixed (chunks start at multiples
  // of 64 rows and RPP is a multiple of 4, so row % 4 == s_r % 4)
  constexpr int ST = WT == kWtTiled ? DT_F16 : WT;        // type of the values as they arrive for staging
  const int tl_ntn = (G.N + 127) / 128, tl_n = (n0 + s_c) & 127;
  const int tl_col = ((n0 + s_c) >> 7) * kTileImageBytes + ((((tl_n >> 5) ^ (s_r & 3)) << 5) + (tl_n & 31)) * 2;
  const int trA = tr_lane_off(lane, WS) + 32 * g * WS;   // transposing-read base of this lane (halves)

  f16v acc[2][NT];
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = zero16();

  RawAct<AM> rawA[2][4];      // [row tile][step]; a slot is refilled right after its last use with the next chunk's data
  u4 w_raw[NP];

  // Operand and weight requests never branch: past the last chunk the resource has size 0 and the loads return zeros
  // (a conditional request inside the MFMA loop would split it into basic blocks with conservative waits).
  auto load_a = [&](int c, int kk, bool live) {
    const int kleft = K - c * kChunkK;
    const rsrc_t r = (AM == AM_FM) ? rsrc_at(a.A, live ? a_total : 0, (long long)c * kFmChunkBytes)
                                   : rsrc_at(a.A, live ? a_total : 0, (long long)c * kChunkK * ESZ);
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      if constexpr (AM == AM_FM) {
        rawA[mt][kk].v = buf_load16(r, voffA[mt] + kk * kFmStepBytes);   // the k padding of an FM tensor holds zeros
      } else {
        const int v = (32 * g + 8 * kk < kleft) ? voffA[mt] : kOobOffset;
        if constexpr (AM == AM_ROW_F32) {
          rawA[mt][kk].lo = buf_load16(r, v + kk * 32);
          rawA[mt][kk].hi = buf_load16(r, v + kk * 32 + 16);
        } else {
          rawA[mt][kk].v = buf_load16(r, v + kk * 16);
        }
      }
    }
  };
  auto w_rsrc = [&](int c, bool live) {
    if constexpr (WT == kWtTiled) {
      const int kt = c >> 1;                              // chunk c = rows 64 (c % 2) .. of tile row c / 2 (zero-padded past K)
      return rsrc_at(G.W, live ? w_total : 0, (long long)kt * tl_ntn * kTileImageBytes + (c & 1) * 64 * 256);
    } else {
      return rsrc_at(G.W, live ? w_total : 0, ((long long)c * kChunkK * G.ldw + n0) * 2);
    }
  };
  auto load_w_pass = [&](const rsrc_t& r, int p) {
    const int off = WT == kWtTiled ? (s_r + p * RPP) * 256 + tl_col : ((s_r + p * RPP) * G.ldw + s_c) * 2;
    w_raw[p] = buf_load16(r, s_ok ? off : kOobOffset);   // rows past K: out of range -> 0
  };
  auto store_w_pass = [&](int buf, int p) { stage_store16<ST>(&lds[buf][(s_r + p * RPP) * WS + s_c], w_raw[p]); };
  auto bias_f4 = [&](u2 raw) -> f4v {
    if constexpr (WT == kWtTiled) return a.w_dt == DT_BF16 ? raw_to_f4<DT_BF16>(raw) : raw_to_f4<DT_F16>(raw);
    else return raw_to_f4<WT>(raw);
  };
  // prologue: chunk 0 in LDS and in the operand registers, chunk 1's weights in flight
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) load_a(cb, kk, cb < ce);
  {
    const rsrc_t r0 = w_rsrc(cb, cb < ce), r1 = w_rsrc(cb + 1, cb + 1 < ce);
#pragma unroll
    for (int p = 0; p < NP; ++p) load_w_pass(r0, p);
#pragma unroll
    for (int p = 0; p < NP; ++p) { store_w_pass(0, p); load_w_pass(r1, p); }
  }
  __syncthreads();
  for (int c = cb; c < ce; ++c) {
    // chunk c+1 (requested during the previous iteration) is stored to the other buffer and chunk c+2 is requested, one
    // staging pass per MFMA step; the activation operands of a step are refilled with chunk c+1's right after their use
    const rsrc_t rw2 = w_rsrc(c + 2, c + 2 < ce);
    const bool more1 = c + 1 < ce;
    const _Float16* wt = lds[(c - cb) & 1];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      h8 bf[NT], af[2];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const _Float16* q = wt + trA + 8 * kk * WS + 32 * nt;
        bf[nt] = tr_frag(q, q + 4 * WS);
      }
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) af[mt] = cvt_raw_act<AM>(rawA[mt][kk]);
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = mfma32(bf[nt], af[mt], acc[mt][nt]);   // rows n, cols tokens
      load_a(c + 1, kk, more1);
      if ((kk * NP) % 4 == 0) {
        const int p = kk * NP / 4;
        store_w_pass((c + 1 - cb) & 1, p);
        load_w_pass(rw2, p);
      }
    }
    __syncthreads();
  }

  // ---- epilogue
  if constexpr (CFM) {
    // lane = token, registers = 4 consecutive output columns: 8-byte stores into the fragment-major output
    const int nch = (G.N + 63) / 64;
    const rsrc_t rB = rsrc_at(G.bias, G.bias ? (long long)G.N * 2 : 0, 0);
    _Float16* C = (_Float16*)G.C;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const int n = n0 + 32 * nt + 8 * jj + 4 * g;   // first of 4 columns
        if (n >= nch * 64) continue;                   // columns N .. 64*nch-1 are written as zeros (FM padding)
        const f4v bias = bias_f4(buf_load8(rB, n * 2));
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
          const int tok = m0 + 32 * mt + l32;
          if (tok < T) {
            const size_t unit = ((size_t)((tok >> 5) * nch + (n >> 6)) * 4 + jj) * 64 + ((n >> 5) & 1) * 32 + (tok & 31);
            h4 o;
#pragma unroll
            for (int i = 0; i < 4; ++i) o[i] = (_Float16)(acc[mt][nt][4 * jj + i] + bias[i]);
            *(h4*)(C + unit * 8 + 4 * g) = o;
          }
        }
      }
  } else if (ksplit > 1) {
    // partial sums [part of the contraction][token][all groups' columns], fp32; bias and residual are added by the reduction
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        const int tok = m0 + 32 * mt + l32;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const int n = n0 + 32 * nt + 8 * jj + 4 * g;
          if (tok < T && n < G.N) {
            f4v x;
#pragma unroll
            for (int i = 0; i < 4; ++i) x[i] = acc[mt][nt][4 * jj + i];
            *(f4v*)(a.part + ((size_t)ks * T + tok) * a.ldp + goff + n) = x;
          }
        }
      }
  } else {
    // row-major output: lane = token, registers = 4 consecutive output columns -> one 16-byte (fp32) or 8-byte store
    const rsrc_t rB = rsrc_at(G.bias, G.bias ? (long long)G.N * 2 : 0, 0);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      f4v bias[4];
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) bias[jj] = bias_f4(buf_load8(rB, (n0 + 32 * nt + 8 * jj + 4 * g) * 2));   // past N: 0
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        const int tok = m0 + 32 * mt + l32;
        // all residual values of the tile are requested before the first store: the output may alias the residual
        // (in-place update of the residual stream), so a load placed after a store would have to wait for it
        f4v res[4];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const int n = n0 + 32 * nt + 8 * jj + 4 * g;
          res[jj] = (a.R && tok < T && n < G.N) ? load4(a.R, (size_t)tok * a.ldr + n, a.r_dt) : f4v{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const int n = n0 + 32 * nt + 8 * jj + 4 * g;
          if (tok < T && n < G.N) {
            f4v x;
#pragma unroll
            for (int i = 0; i < 4; ++i) x[i] = acc[mt][nt][4 * jj + i] + bias[jj][i] + res[jj][i];
            store4(G.C, (size_t)tok * G.ldc + n, x, a.c_dt);
          }
        }
      }
    }
  }
}

// sum of the partial results over the parts of the contraction (fixed order) + bias + residual -> row-major output
__global__ void __launch_bounds__(256) linear_reduce_kernel(LinearArgs a, int ksplit) {
  const int quads = a.ldp / 4;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)a.T * quads) return;
  const int tok = (int)(i / quads);
  int n = 4 * (int)(i % quads), gi = 0;
  for (; gi < a.ngroups - 1 && n >= a.g[gi].N; ++gi) n -= a.g[gi].N;
  const LinearGroup G = a.g[gi];
  f4v x = {0.f, 0.f, 0.f, 0.f};
  for (int ks = 0; ks < ksplit; ++ks) {
    const f4v p = *(const f4v*)(a.part + ((size_t)ks * a.T + tok) * a.ldp + 4 * (i % quads));
#pragma unroll
    for (int e = 0; e < 4; ++e) x[e] += p[e];
  }
  if (G.bias) {
    const f4v b = load4(G.bias, n, a.w_dt);
#pragma unroll
    for (int e = 0; e < 4; ++e) x[e] += b[e];
  }
  if (a.R) {
    const f4v r = load4(a.R, (size_t)tok * a.ldr + n, a.r_dt);
#pragma unroll
    for (int e = 0; e < 4; ++e) x[e] += r[e];
  }
  store4(G.C, (size_t)tok * G.ldc + n, x, a.c_dt);
}

template <int AM, int WT, bool CFM>
hipError_t launch_bn(const LinearArgs& a, hipStream_t s) {
  const int tiles_m = (a.T + 255) / 256;
  int n128 = 0, n64 = 0;
  for (int i = 0; i < a.ngroups; ++i) { n128 += (a.g[i].N + 127) / 128; n64 += (a.g[i].N + 63) / 64; }
  // narrow tiles when the wide ones would leave compute units idle or unevenly loaded (two wide or four narrow
  // workgroups fit on a compute unit)
  const bool narrow = (long)tiles_m * n128 < 512;
  // one tile row and room for partial sums: split the contraction so that about one workgroup per compute unit runs
  int ksplit = 1;
  if (!CFM && a.part && tiles_m == 1 && a.ldp > 0) {
    const int kchunks = (a.K + kChunkK - 1) / kChunkK;
    const size_t room = a.part_bytes / ((size_t)a.T * a.ldp * 4);
    ksplit = 256 / n64;
    if (ksplit > kchunks / 2) ksplit = kchunks / 2;          // at least two 64-wide chunks per part
    if ((size_t)ksplit > room) ksplit = (int)room;
    if (ksplit < 1 || !narrow) ksplit = 1;
  }
  if (narrow) {
    hipLaunchKernelGGL((linear_kernel<AM, WT, 64, CFM>), dim3(tiles_m * n64 * ksplit), dim3(256), 0, s, a, tiles_m, n64, ksplit);
  } else {
    hipLaunchKernelGGL((linear_kernel<AM, WT, 128, CFM>), dim3(tiles_m * n128), dim3(256), 0, s, a, tiles_m, n128, 1);
  }
  if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
  if (ksplit > 1) {
    const size_t quads = (size_t)a.T * (a.ldp / 4);
    hipLaunchKernelGGL(linear_reduce_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, s, a, ksplit);
  }
  return hipGetLastError();
}

template <int AM, int WT>
hipError_t launch_c(const LinearArgs& a, hipStream_t s) {
  return a.c_layout == LAYOUT_FM ? launch_bn<AM, WT, true>(a, s) : launch_bn<AM, WT, false>(a, s);
}

template <int WT>
hipError_t launch_a(const LinearArgs& a, hipStream_t s) {
  if (a.a_layout == LAYOUT_FM) return launch_c<AM_FM, WT>(a, s);
  if (a.a_dt == DT_F16) return launch_c<AM_ROW_F16, WT>(a, s);
  if (a.a_dt == DT_BF16) return launch_c<AM_ROW_BF16, WT>(a, s);
  return launch_c<AM_ROW_F32, WT>(a, s);
}

}  // namespace

hipError_t launch_linear(const LinearArgs& a, hipStream_t s) {
  if (a.w_tiled) return launch_a<kWtTiled>(a, s);
  return a.w_dt == DT_F16 ? launch_a<DT_F16>(a, s) : launch_a<DT_BF16>(a, s);
}

}  // namespace fsvd
