// Host-side launch interface of the fsvd kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace fsvd {

// ---- C[T, N] = A[T, K] W[K, N] (+ bias[N]) (+ R[T, N]) for up to three weight matrices sharing A
struct LinearGroup {
  const void* W;     // [K, N] row-major, stored in w_dt
  const void* bias;  // [N] in w_dt, or nullptr
  void* C;           // [T, N] with row stride ldc
  int N;
  int ldw;
  int ldc;
};
struct LinearArgs {
  const void* A;  // [T, K] row stride lda, stored in a_dt (F16, BF16 or F32)
  int lda;
  int a_dt;
  int T;
  int K;
  int w_dt;       // F16 or BF16
  int c_dt;       // F16, BF16 or F32
  const void* R;  // residual added in the epilogue (group 0 indexing), or nullptr
  int ldr;
  int r_dt;
  int ngroups;
  LinearGroup g[3];
};
hipError_t launch_linear(const LinearArgs& a, hipStream_t s);

// ---- streaming attention core (Alg. 1 Part II): rank-space P_q, P_k, P_v -> context C [T, D] (fp16)
struct AttnCoreArgs {
  const _Float16* Pq; const _Float16* Pk; const _Float16* Pv;  // [B*M, r_x], row strides ldpq/ldpk/ldpv
  int ldpq, ldpk, ldpv;
  int rq, rk, rv;
  const void* Vq; const void* Vk; const void* Vv;   // [r_x, D] stored in w_dt
  const void* bq; const void* bk; const void* bv;   // [D] in w_dt or nullptr
  int w_dt;
  int B, M, D, H;
  int causal;
  const int32_t* key_len;  // device [B] or nullptr
  float scale;             // softmax scale (already resolved, > 0)
  _Float16* C;             // [B*M, D]
  int ldc;
};
hipError_t launch_attn_core(const AttnCoreArgs& a, hipStream_t s);

// ---- fused FFN core (Alg. 2 inner loops): P1 [T, r1] -> Z [T, r2] = phi(P1 V1 + b1) U2
struct FfnCoreArgs {
  const _Float16* P1; int ldp; int r1;
  const void* V1;    // [r1, F] in w_dt
  const void* b1;    // [F] in w_dt or nullptr
  const void* U2;    // [F, r2] in w_dt
  int r2;
  int w_dt;
  int T, F;
  int act;
  _Float16* Z; int ldz;  // [T, r2]
};
hipError_t launch_ffn_core(const FfnCoreArgs& a, hipStream_t s);

// ---- LayerNorm over the last axis of [T, D]; writes up to two copies
struct LayerNormArgs {
  const void* X; int x_dt; int ldx;   // input in F16 / BF16 / F32
  const void* gamma; const void* beta; int p_dt;
  float eps;
  int T, D;
  void* Y0; int y0_dt; int ldy0;      // first output (required)
  void* Y1; int y1_dt; int ldy1;      // optional second copy (nullptr to skip)
};
hipError_t launch_layernorm(const LayerNormArgs& a, hipStream_t s);

}  // namespace fsvd
