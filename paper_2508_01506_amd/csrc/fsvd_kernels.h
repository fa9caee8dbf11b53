// Host-side launch interface of the fsvd kernels (internal to the library).
//
// "FM" below is the fragment-major fp16 activation layout defined in fsvd_common.h: every
// intermediate activation that feeds a matrix-core contraction is kept in it.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace fsvd {

enum : int { LAYOUT_ROW = 0, LAYOUT_FM = 1 };

// ---- C[T, N] = A[T, K] W[K, N] (+ bias[N]) (+ R[T, N]) for up to three weight matrices sharing A
struct LinearGroup {
  const void* W;     // [K, N] row-major, stored in w_dt; or its tile images (LinearArgs::w_tiled)
  const void* bias;  // [N] in w_dt, or nullptr
  void* C;           // ROW: [T, N] with row stride ldc; FM: fragment-major [T, N] (fp16)
  int N;
  int ldw;
  int ldc;
};
struct LinearArgs {
  const void* A;  // ROW: [T, K] row stride lda in a_dt (F16, BF16 or F32); FM: fragment-major fp16 [T, K]
  int a_layout;
  int lda;
  int a_dt;
  int T;
  int K;
  int w_dt;       // F16 or BF16 (bias; and W unless w_tiled)
  int w_tiled;    // non-zero: every group's W is a prepacked fp16 tile image of [K, N] (ldw unused)
  int c_layout;   // LAYOUT_ROW or LAYOUT_FM
  int c_dt;       // ROW only: F16, BF16 or F32
  const void* R;  // ROW only: residual [T, N] row stride ldr, added in the epilogue, or nullptr
  int ldr;
  int r_dt;
  int ngroups;
  LinearGroup g[3];
  // optional, row-major output and T <= 256 only: room for fp32 partial sums [parts][T][ldp] when the contraction is
  // split over workgroups (ldp = sum of the groups' N); nullptr = never split
  float* part;
  size_t part_bytes;
  int ldp;
};
hipError_t launch_linear(const LinearArgs& a, hipStream_t s);

// ---- Y = LN(A W + bias + R) in one kernel (fsvd_gemm_ln.hip): A fragment-major fp16 [T, K], W tile images of [K, D]
struct LinearLnArgs {
  const void* A; int T, K, D;
  const void* W;                       // prepacked tile images of [K, D]
  const void* bias; int w_dt;          // [D] in w_dt or nullptr
  const void* R; int r_dt;             // residual [T, D] row-major or nullptr
  const void* gamma; const void* beta; int p_dt;
  float eps;
  void* Yrow; int yrow_dt;             // row-major output or nullptr (may alias R: every row is read before it is written)
  void* Yfm;                           // fragment-major fp16 output or nullptr
};
bool linear_ln_supported(int D);
bool linear_ln_fits(long long T, int D);   // [T, D] small enough for the kernel's 32-bit offsets
hipError_t launch_linear_ln(const LinearLnArgs& a, hipStream_t s);

// ---- streaming attention core (Alg. 1 Part II): FM P_q, P_k, P_v -> FM context C [T, D]
struct AttnCoreArgs {
  const void* Pq; const void* Pk; const void* Pv;   // FM [B*M, r_x] (grouped factors: [B*M, G * r_x], group g = columns g r_x ..)
  int rq, rk, rv;
  int per_head;            // 0: whole-matrix factors, V_x [r_x, D]; n >= 1: grouped factors with n heads per group,
                           // V_x [H / n, r_x, n d_h] (n = 1: one pair per head)
  const void* Vq; const void* Vk; const void* Vv;   // stored in w_dt
  const void* bq; const void* bk; const void* bv;   // [D] in w_dt or nullptr
  int w_dt;
  int tiled;               // non-zero: Vq, Vk, Vv are prepacked fp16 tile images of [r_x, D] (whole-matrix factors only)
  int B, M, D, H;
  int causal;
  const int32_t* key_len;  // device [B] or nullptr
  float scale;             // softmax scale (already resolved, > 0)
  void* C;                 // FM [B*M, D]
};
hipError_t launch_attn_core(const AttnCoreArgs& a, hipStream_t s);
// the absorbed schedule for one factor pair per head with ranks <= 64 (fsvd_attn_absorbed.hip): no K / V rebuild
bool attn_absorbed_supported(const AttnCoreArgs& a);
hipError_t launch_attn_absorbed(const AttnCoreArgs& a, hipStream_t s);

// ---- fused FFN core (Alg. 2 inner loops): FM P1 [T, r1] -> FM Z [T, r2] = phi(P1 V1 + b1) U2
struct FfnCoreArgs {
  const void* P1; int r1;
  const void* V1;    // [r1, F] in w_dt
  const void* b1;    // [F] in w_dt or nullptr
  const void* U2;    // [F, r2] in w_dt
  int r2;
  int w_dt;
  int tiled;         // non-zero: V1 and U2 are prepacked fp16 tile images (b1 stays in w_dt)
  int T, F;
  int act;
  void* Z;           // [T, r2] fragment-major fp16
  float* Zpart;      // fp32 partial sums, FfnCorePlan::partial_bytes (needed when the plan splits F)
};
// launch shape of the FFN core for a problem size (host-side, no device needed)
// wide > 0: the all-wavefront kernel for prepacked weights (fsvd_ffn_wide.hip) with `wide` 256-rank groups per workgroup
// (slice_w = 256 wide); wide == 0: the two-role kernel (fsvd_ffn.hip) with ns + ns2 128-rank sub-tiles per workgroup
struct FfnCorePlan { int nslices, slice_w, ns, ns2, fsplit, wide; size_t partial_bytes; };
FfnCorePlan ffn_core_plan(int T, int r1, int r2, int F, bool tiled);
hipError_t launch_ffn_core(const FfnCoreArgs& a, hipStream_t s);
hipError_t launch_ffn_core_wide(const FfnCoreArgs& a, const FfnCorePlan& pl, hipStream_t s);

// ---- whole factored FFN in one kernel (Alg. 3): row-major X [T, D] -> row-major out [T, D], no intermediates in memory
struct FfnV2Args {
  const void* X; int x_dt;                // [T, D] row-major
  const void *U1, *V1, *U2, *V2;          // prepacked fp16 tile images of [D, r1], [r1, F], [F, r2], [r2, D]
  const void *b1, *b2; int w_dt;          // [F], [D] in w_dt or nullptr
  int T, D, F, r1, r2, act;
  void* out; int out_dt;                  // [T, D] row-major
};
bool ffn_v2_supported(int D, int F, int r1, int r2);
hipError_t launch_ffn_v2(const FfnV2Args& a, hipStream_t s);

// ---- decoding step against a rank-space KV cache (layouts and kernels: fsvd_decode.hip)
inline size_t decode_vcache_seq_bytes(size_t t_max, size_t r_v) { return ((t_max + 31) / 32) * ((r_v + 31) / 32) * 2048; }
struct DecodeCoreArgs {
  const void* W;          // absorbed queries, per sequence the fragment-major layout of [32, r_k] (fp16)
  const void* kcache;     // per sequence: fragment-major P_k [t_max, r_k]
  const void* vcache;     // per sequence: P_v^T in operand order (decode_vcache_seq_bytes)
  const int32_t* n_keys;  // device [B]: valid keys of each sequence
  int B, t_max, r_k, r_v, nsplit;
  float* stats;           // [B * nsplit slots][64]: running maximum (32 heads) | sum (32 heads); slot = workgroup
  _Float16* upart;        // [B * nsplit slots][r_v][32 heads]: U / l
};
hipError_t launch_decode_cache_write(const void* src, const int32_t* t_start, int B, int t_max, int r, int n_new, int which,
                                     void* cache, hipStream_t s);
hipError_t launch_decode_absorb(const void* q, const void* Vk, int w_dt, int B, int D, int H, int r_k, float scale, void* W,
                                hipStream_t s);
hipError_t launch_decode_core(const DecodeCoreArgs& a, hipStream_t s);
hipError_t launch_decode_merge(const float* stats, const void* upart, const int32_t* n_keys, int B, int t_max, int nsplit, int H, int r_v,
                               float* u_out, hipStream_t s);
hipError_t launch_decode_value(const float* u, const void* Vv, const void* bv, int w_dt, int B, int D, int H, int r_v, void* ctx,
                               hipStream_t s);
hipError_t launch_decode_append(const void* pk, const void* pv, const int32_t* t_len, int B, int t_max, int r_k, int r_v,
                                void* kcache, void* vcache, int32_t* n_keys, hipStream_t s);

// ---- LayerNorm over the last axis of a row-major [T, D]; writes a row-major copy and/or an FM copy
struct LayerNormArgs {
  const void* X; int x_dt;            // row-major, F16 / BF16 / F32
  const void* gamma; const void* beta; int p_dt;
  float eps;
  int T, D;
  void* Yrow; int yrow_dt;            // row-major output or nullptr
  void* Yfm;                          // FM fp16 output or nullptr
};
hipError_t launch_layernorm(const LayerNormArgs& a, hipStream_t s);

// ---- weight prepacking: row-major [K, N] (F16 / BF16) -> fp16 tile images (tiled_bytes(K, N) bytes)
hipError_t launch_pack_tiled(const void* src, int src_dt, int K, int N, void* dst, hipStream_t s);

// ---- layout conversion: row-major [T, K] (F16 / BF16 / F32) <-> FM fp16
hipError_t launch_pack_fm(const void* src, int src_dt, int T, int K, void* dst_fm, hipStream_t s);
hipError_t launch_unpack_fm(const void* src_fm, int T, int K, void* dst, int dst_dt, hipStream_t s);

// ---- matrix-core rate probe: workgroups x 4 wavefronts, each iters x 4 MFMAs (32x32x16 fp16) on registers;
// out: float[workgroups * 256]
hipError_t launch_mfma_probe(int workgroups, int iters, float* out, hipStream_t s);
// ---- L2 -> LDS delivery probe: workgroups x `steps` steps of 32 KiB copied straight into LDS from one of eight regions
// of `region_bytes` (a multiple of 32 KiB) of src; out: float[workgroups * 512]
hipError_t launch_dma_probe(int workgroups, int steps, int with_work, const void* src, unsigned region_bytes, float* out, hipStream_t s);

}  // namespace fsvd
