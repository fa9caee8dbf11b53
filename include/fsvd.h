/*
 * fsvd — rank-aware streaming execution of one SVD-compressed transformer layer
 * on AMD MI355X (gfx950).  C ABI.
 *
 * Every projection matrix W [in, out] of the layer is given as a rank-r factor
 * pair W ~= U V with U [in, r], V [r, out] and a dense bias b [out]
 * (Methodology, "Optimal Low-Rank Factorization via SVD": W^[r] = U~ V~^T with
 * the singular values split evenly into both factors).  The library evaluates
 * the layer so that the full-width intermediates — the [B*M, D] query, key and
 * value tensors, the [B, H, M, M] scores and the [B*M, F] FFN hidden
 * activation — are rebuilt tile by tile on chip and never written to device
 * memory; only rank-space tensors ([B*M, r]) and model-width block
 * inputs/outputs ([B*M, D]) pass through the caller's workspace.
 *
 * Conventions shared by all entry points
 *  - Pointers.  Every data pointer (X, factors, biases, LayerNorm parameters,
 *    key_len, out, workspace) is a DEVICE pointer owned by the caller and only
 *    borrowed for the duration of the call.  The descriptor and fsvd_factor
 *    structs themselves are HOST memory.  The library never allocates or frees
 *    device memory and keeps no state between calls; all scratch is carved
 *    from `workspace`, which must be 256-byte aligned and at least as large as
 *    the matching fsvd_*_workspace() value.  The transient activation memory
 *    of a call is therefore exactly `workspace_bytes`.  Every other data
 *    pointer must be 16-byte aligned (FSVD_ERR_INVALID_ARG otherwise).
 *    Calls on one stream may share a workspace; calls that overlap in time
 *    need workspaces of their own.
 *  - Layouts.  Row-major, contiguous.  X and out are [B, M, D]; U is
 *    [in, rank]; V is [rank, out]; bias is [out] (or NULL for no bias).  Head h
 *    of an attention projection owns output columns [h*d_h, (h+1)*d_h) of V,
 *    d_h = D / H (Definition "Attention Activation Approximation").
 *  - Types.  X, U, V, bias, gamma and beta are stored in `io_dtype` (FSVD_F16
 *    or FSVD_BF16).  All contractions run on the fp16 matrix cores with fp32
 *    accumulation; bf16 inputs are widened to fp16 on load, which is exact for
 *    2^-14 <= |x| <= 65504 (the range precondition of bf16 models).  Outside
 *    it nothing is reported and the behaviour is: a bf16 element of X, U or
 *    V (row-major or through fsvd_pack_tiled) is converted with rounding
 *    toward zero, so |x| > 65504 saturates to +-65504 (never to infinity) and
 *    |x| < 2^-14 is truncated to fp16's subnormal grid (spacing 2^-24; below
 *    2^-24 it becomes 0).  Biases and LayerNorm parameters are used as fp32
 *    and have no such limit; fp16 hand-offs between the kernels (rank-space
 *    activations, context) round to nearest and can overflow to infinity if
 *    such inputs drive them beyond 65504.  `out` is written in `out_dtype`
 *    (FSVD_F16, FSVD_BF16 or FSVD_F32).
 *  - Streams.  All work is enqueued on `hip_stream` (a hipStream_t passed as
 *    void*; NULL is the default stream).  No call synchronises the host.
 *  - Errors.  Arguments are validated before anything is launched; a call
 *    either enqueues the whole computation and returns FSVD_OK or enqueues
 *    nothing and returns an error code.  Nothing aborts or throws.  The
 *    *_workspace() functions return 0 for an invalid descriptor.
 *  - Limits.  D % H == 0 and d_h in {64, 128}; D, F and every rank are
 *    multiples of 16 (a rank that is not can be zero-padded by the caller,
 *    which leaves the result unchanged: Alg. 1 Part I pads the rank the same
 *    way); B*M*max(D, F) < 2^29 and every tensor smaller than 2 GiB;
 *    key_len[b] in [1, M].
 */
#ifndef FSVD_H
#define FSVD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FSVD_OK = 0,
  FSVD_ERR_INVALID_ARG = 1,  /* null pointer, non-positive size, inconsistent factor shapes */
  FSVD_ERR_UNSUPPORTED = 2,  /* valid request outside the supported limits listed above */
  FSVD_ERR_WORKSPACE = 3,    /* workspace NULL, misaligned or too small */
  FSVD_ERR_DEVICE = 4        /* a HIP launch failed; hipGetLastError() has the detail */
} fsvd_status;

typedef enum { FSVD_F16 = 0, FSVD_BF16 = 1, FSVD_F32 = 2 } fsvd_dtype;
typedef enum { FSVD_ACT_GELU_ERF = 0, FSVD_ACT_GELU_TANH = 1, FSVD_ACT_RELU = 2 } fsvd_act;
typedef enum { FSVD_NORM_NONE = 0, FSVD_NORM_POST_LN = 1, FSVD_NORM_PRE_LN = 2 } fsvd_norm;

/* How a factor matrix is stored.  ROW_MAJOR: as described under "Layouts", in io_dtype.  TILED: prepacked once by
 * fsvd_pack_tiled (at model load) into fp16 tile images that the kernels copy into on-chip memory byte for byte;
 * see fsvd_pack_tiled for the format and for which matrices may be given this way. */
typedef enum { FSVD_ROW_MAJOR = 0, FSVD_TILED = 1 } fsvd_layout;

/* One factored projection W ~= U V (+ bias).  U [in_dim, rank], V [rank, out_dim],
 * bias [out_dim] or NULL; device pointers in the descriptor's io_dtype (bias always; U and V unless
 * their layout member says FSVD_TILED).  A zero-initialised u_layout / v_layout means row-major. */
typedef struct {
  const void *U;
  const void *V;
  const void *bias;
  int32_t in_dim;
  int32_t rank;
  int32_t out_dim;
  int32_t u_layout;   /* fsvd_layout of U */
  int32_t v_layout;   /* fsvd_layout of V */
  int32_t groups;     /* only read by the *_heads entry points: number of head groups G (0 = one group per head) */
} fsvd_factor;

/* Problem descriptor (host memory). */
typedef struct {
  int32_t B;             /* sequences */
  int32_t M;             /* tokens per sequence */
  int32_t D;             /* model width */
  int32_t H;             /* attention heads, d_h = D / H */
  int32_t F;             /* FFN hidden width (ignored by fsvd_attention) */
  fsvd_dtype io_dtype;   /* storage type of X and of all parameters: F16 or BF16 */
  fsvd_dtype out_dtype;  /* type of `out`: F16, BF16 or F32 */
  int32_t causal;        /* non-zero: key j is visible to query i only if j <= i */
  const int32_t *key_len;/* device int32[B] or NULL: keys j >= key_len[b] are masked for every
                            query of sequence b (all M query rows are still computed) */
  float softmax_scale;   /* 0 selects 1/sqrt(d_h) (Alg. 1 Part II) */
  fsvd_act act;          /* FFN non-linearity phi */
  fsvd_norm norm;        /* residual / LayerNorm wiring of fsvd_layer */
  float ln_eps;          /* LayerNorm epsilon (biased variance) */
} fsvd_desc;

/* Workspace sizes in bytes (multiples of 256); 0 if the request is invalid or unsupported.
 * Pure host functions: they touch no device. */
size_t fsvd_attention_workspace(const fsvd_desc *desc, int32_t r_q, int32_t r_k, int32_t r_v, int32_t r_o);
size_t fsvd_ffn_workspace(const fsvd_desc *desc, int32_t r_1, int32_t r_2);
size_t fsvd_layer_workspace(const fsvd_desc *desc, int32_t r_q, int32_t r_k, int32_t r_v, int32_t r_o,
                            int32_t r_1, int32_t r_2);

/* Validation only (what the compute entry points run before launching); touches no device.
 * Useful to check a configuration without a GPU. */
fsvd_status fsvd_attention_check(const fsvd_desc *desc, const fsvd_factor *q, const fsvd_factor *k,
                                 const fsvd_factor *v, const fsvd_factor *o);
fsvd_status fsvd_ffn_check(const fsvd_desc *desc, const fsvd_factor *w1, const fsvd_factor *w2);

/*
 * Attention block, FlashSVDAttention (Alg. 1; section "FlashSVDAttention"):
 *   P_a = X U_a for a in {q, k, v}                       (rank space, workspace)
 *   per (sequence, head, query block): rebuild Q = P_q V_q[:, head] + b_q on chip; for every
 *   key block rebuild K and V the same way, scores = Q K^T * softmax_scale, masks,
 *   streaming softmax, context += alpha V                (Alg. 1 Part I + II)
 *   out = (context U_o) V_o + b_o                        (output projection in factored form)
 * X [B, M, D] -> out [B, M, D].  q, k, v, o: in_dim = out_dim = D, ranks free.
 */
fsvd_status fsvd_attention(const fsvd_desc *desc, const void *X, const fsvd_factor *q, const fsvd_factor *k,
                           const fsvd_factor *v, const fsvd_factor *o, void *out, void *workspace,
                           size_t workspace_bytes, void *hip_stream);

/*
 * The same attention block with PER-HEAD factors of q, k and v, the setting Alg. 1 is written in (V_a in
 * R^{r x d_h} per head; appendix on multi-head low-rank activations): head h of projection a has its own pair
 * U_a^(h) [D, r_a], V_a^(h) [r_a, d_h].  For q, k, v the fsvd_factor members then mean: `rank` = r_a of ONE head;
 * U = [U^(1) | ... | U^(H)], row-major [D, H * rank]; V = the H matrices V^(h) one after another, [H, rank, d_h];
 * bias [D] as before (head h owns entries h*d_h ..); in_dim = out_dim = D.  o stays a whole-matrix factor.
 * The rank-space activations P_a are [B*M, H * rank]; a head's K and V tiles are rebuilt from its own block of
 * r_a ranks, so the on-chip rebuild costs 2 * r_a * d_h FLOPs per key and tile instead of 2 * r * d_h with a
 * whole-matrix rank r.  Ranks are multiples of 16 (r_a <= d_h is the intended range, larger values work).
 * With one pair per head and all three ranks <= 64 the core runs Alg. 1's schedule for r <= d_h with everything
 * absorbed: M_h = V_q^(h) V_k^(h)^T once per workgroup, w = scale * (P_q^(h) M_h + b_q^(h) V_k^(h)^T), scores
 * w . P_k^(h)[key] contracted over r_k (the q . b_k term is constant per row and cancels in the softmax), the
 * context accumulated in rank space as u = softmax . P_v^(h) and projected once, u V_v^(h) + b_v^(h).  No Q, K or V
 * tile exists, on chip or off; the fp16 hand-offs are then M_h, w, the probabilities and u.  The environment
 * variable FSVD_ATTN_ABSORBED=0, read at every call, keeps the rebuilding schedule for such factors (a switch for
 * comparisons; both meet the same tolerances).
 * Same conventions, limits and errors as fsvd_attention; additionally H * rank * D < 2^29.
 *
 * Grouped heads (appendix, grouped-head compression): with `groups` = G (a divisor of H, the same for q, k, v) the
 * heads are compressed jointly in G groups of H / G consecutive heads; `rank` is then the rank of ONE group,
 * U = [U^(1) | ... | U^(G)] [D, G * rank] and V = [G, rank, D / G] (group g's pair rebuilds the columns of its heads).
 * G = H (or 0) is the per-head layout above, G = 1 computes the same as fsvd_attention.  The workspace of a grouped
 * call is sized by the *_groups_workspace functions (the *_heads_workspace functions are the case G = H).
 */
size_t fsvd_attention_heads_workspace(const fsvd_desc *desc, int32_t r_q, int32_t r_k, int32_t r_v, int32_t r_o);
size_t fsvd_attention_groups_workspace(const fsvd_desc *desc, int32_t groups, int32_t r_q, int32_t r_k, int32_t r_v,
                                       int32_t r_o);
fsvd_status fsvd_attention_heads(const fsvd_desc *desc, const void *X, const fsvd_factor *q, const fsvd_factor *k,
                                 const fsvd_factor *v, const fsvd_factor *o, void *out, void *workspace,
                                 size_t workspace_bytes, void *hip_stream);

/*
 * Feed-forward block, FlashSVDFFN V1 (Alg. 2; section "FlashSVDFFN V1"):
 *   P = X U_1                                            (rank space, workspace)
 *   per row block, streaming over F: Y = phi(P V_1[:, chunk] + b_1[chunk]) on chip,
 *   Z += Y U_2[chunk, :]                                 (rank space, workspace)
 *   out = Z V_2 + b_2
 * X [B, M, D] -> out [B, M, D].  w1: D -> F, w2: F -> D.
 */
fsvd_status fsvd_ffn(const fsvd_desc *desc, const void *X, const fsvd_factor *w1, const fsvd_factor *w2,
                     void *out, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * fsvd_ffn for callers that cannot allocate device memory or hand over a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid allocation.  Same arguments, checks, kernels and results (bit for bit)
 * as fsvd_ffn, but the rank-space scratch (P, Z and, when the core splits the sum over F, its fp32 partial sums)
 * lives in an array of FSVD_STATIC_SCRATCH_BYTES that is part of the library's device image: every GPU the library
 * runs on holds its own copy from the moment the library is loaded there until the process ends.  The call
 * allocates and frees nothing (no hipMalloc, hipFree or allocating runtime routine); on its first use on a device it
 * looks the array's address up once (hipGetSymbolAddress, with that device current) and keeps it per device.
 * The device that is current when the call is made must be the one hip_stream and all pointers belong to.
 * Limit: fsvd_ffn_workspace(desc, w1->rank, w2->rank) <= FSVD_STATIC_SCRATCH_BYTES, otherwise FSVD_ERR_WORKSPACE
 * before any launch (use fsvd_ffn with a caller workspace for larger problems).  Nothing in the scratch has to start
 * at zero (every byte a kernel reads was written earlier in the same call), so the array is never cleared.
 * All calls on one GPU share that GPU's array: calls that may overlap on one GPU (different streams, or host
 * threads without ordering) race on it; calls on one stream are ordered by the stream and may follow one another.
 */
#define FSVD_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
fsvd_status fsvd_ffn_static(const fsvd_desc *desc, const void *X, const fsvd_factor *w1, const fsvd_factor *w2,
                            void *out, void *hip_stream);

/*
 * Feed-forward block, FlashSVDFFN V2 (Alg. 3; section "FlashSVDFFN V2"): the same function as fsvd_ffn,
 *   out = phi((X U_1) V_1 + b_1) U_2 V_2 + b_2,
 * computed by ONE kernel per block of 32 or 64 tokens: the rank projection X U_1 and the up-projection Z V_2 run inside
 * the kernel too, so neither the rank-space activations (P, Z) nor the hidden activation are ever written to device
 * memory and the call needs no workspace.  The price is that every workgroup streams all four factor matrices
 * (they are not reused across as many tokens as in fsvd_ffn), the latency / memory trade the paper reports for V2.
 * X [B, M, D] row-major in io_dtype -> out [B, M, D] in out_dtype; desc->H is not used beyond the common checks.
 * Requirements: U and V of BOTH factors are prepacked tile images (FSVD_TILED, see fsvd_pack_tiled); biases stay in
 * io_dtype (or NULL); ranks are multiples of 16 and at most 1024.  Anything else -> FSVD_ERR_UNSUPPORTED before any
 * launch.  Results agree with fsvd_ffn to the rounding of the fp16 intermediates (P, hidden, Z), which both round the
 * same way.  Device pointers, borrowed for the call; asynchronous on hip_stream.
 */
fsvd_status fsvd_ffn_v2(const fsvd_desc *desc, const void *X, const fsvd_factor *w1, const fsvd_factor *w2,
                        void *out, void *hip_stream);

/*
 * One transformer layer built from the two blocks above.  The residual / LayerNorm wiring is
 * not part of the paper's method (it only notes that these ops remain once the blocks are fused,
 * section "FlashSVDFFN V2"); desc->norm selects
 *   POST_LN: Y1 = LN1(X + Attn(X));      out = LN2(Y1 + FFN(Y1))
 *   PRE_LN : X1 = X + Attn(LN1(X));      out = X1 + FFN(LN2(X1))
 *   NONE   : out = FFN(Attn(X))          (ln*_gamma / ln*_beta may be NULL)
 * LN(x) = gamma (x - mean) / sqrt(var + ln_eps) + beta per token, biased variance, fp32 statistics.
 */
fsvd_status fsvd_layer(const fsvd_desc *desc, const void *X, const fsvd_factor *q, const fsvd_factor *k,
                       const fsvd_factor *v, const fsvd_factor *o, const void *ln1_gamma, const void *ln1_beta,
                       const fsvd_factor *w1, const fsvd_factor *w2, const void *ln2_gamma, const void *ln2_beta,
                       void *out, void *workspace, size_t workspace_bytes, void *hip_stream);

/* The same layer with per-head factors of q, k and v (see fsvd_attention_heads); o, w1, w2 as in fsvd_layer. */
size_t fsvd_layer_heads_workspace(const fsvd_desc *desc, int32_t r_q, int32_t r_k, int32_t r_v, int32_t r_o,
                                  int32_t r_1, int32_t r_2);
size_t fsvd_layer_groups_workspace(const fsvd_desc *desc, int32_t groups, int32_t r_q, int32_t r_k, int32_t r_v,
                                   int32_t r_o, int32_t r_1, int32_t r_2);
fsvd_status fsvd_layer_heads(const fsvd_desc *desc, const void *X, const fsvd_factor *q, const fsvd_factor *k,
                             const fsvd_factor *v, const fsvd_factor *o, const void *ln1_gamma, const void *ln1_beta,
                             const fsvd_factor *w1, const fsvd_factor *w2, const void *ln2_gamma, const void *ln2_beta,
                             void *out, void *workspace, size_t workspace_bytes, void *hip_stream);


/* ------------------------------------------------------------------------------------------
 * Building blocks.  The three entry points above are sequences of these steps; they are exported
 * so that each kernel can be checked and timed on its own.  Same pointer, stream and error
 * conventions; row-major tensors are contiguous (row stride = number of columns); none needs a workspace.
 * ------------------------------------------------------------------------------------------ */

/* C[T, N] = A[T, K] W[K, N] (+ bias[N]) (+ residual[T, N]): the rank projection P = X U, the
 * up-projections (.) V + b and the factored output projection are all this (Alg. 2 "GEMM 1st" and
 * "GEMM 2nd"; FlashSVDAttention text, P_a = X U_a).  a_dtype: F16, BF16 or F32; w_dtype (W and bias):
 * F16 or BF16; residual may be NULL, else it is read in r_dtype; C is written in c_dtype.
 * K and N must be multiples of 16. */
fsvd_status fsvd_linear(int32_t T, int32_t K, int32_t N, const void *A, fsvd_dtype a_dtype, const void *W,
                        const void *bias, fsvd_dtype w_dtype, const void *residual, fsvd_dtype r_dtype,
                        void *C, fsvd_dtype c_dtype, void *hip_stream);

/* fsvd_linear with W given as tile images of [K, N] (fsvd_pack_tiled); bias, if any, in bias_dtype (F16 or BF16). */
fsvd_status fsvd_linear_tiled(int32_t T, int32_t K, int32_t N, const void *A, fsvd_dtype a_dtype, const void *W_tiled,
                              const void *bias, fsvd_dtype bias_dtype, const void *residual, fsvd_dtype r_dtype,
                              void *C, fsvd_dtype c_dtype, void *hip_stream);

/*
 * Fragment-major ("FM") layout.  Inside the library every activation that feeds a matrix-core
 * contraction is fp16 in this layout, and the two kernels below take and return it.  For A [T, K]:
 * tokens are grouped in tiles of 32 and the contraction axis in chunks of 64 (both zero- or
 * garbage-padded); block (tile, chunk) occupies 4 KiB at ((tile * ceil(K/64)) + chunk) * 4096 and holds,
 * for step kk = 0..3, 64 units of 16 bytes: unit kk * 64 + 32 g + (t % 32) stores
 * A[t, 64 chunk + 32 g + 8 kk + 0..7].  fsvd_fm_bytes gives the buffer size (0 if K % 8 != 0);
 * fsvd_pack_fm converts a contiguous row-major [T, K] tensor (F16, BF16 or F32) and zero-fills the
 * padding; fsvd_unpack_fm converts back to row-major (F16, BF16 or F32).
 */
size_t fsvd_fm_bytes(int32_t T, int32_t K);
fsvd_status fsvd_pack_fm(int32_t T, int32_t K, const void *src, fsvd_dtype src_dtype, void *dst_fm, void *hip_stream);
fsvd_status fsvd_unpack_fm(int32_t T, int32_t K, const void *src_fm, void *dst, fsvd_dtype dst_dtype, void *hip_stream);

/*
 * Prepacked weights ("tile images").  The fused kernels stream their weight operands (the V factors that rebuild
 * full-width tiles, Alg. 1 Part I and Alg. 2's inner loops) through on-chip memory in tiles of 128 x 128.  A matrix
 * W [rows, cols] that is constant across calls can be converted once into the exact byte image of those tiles:
 * fp16 (bf16 sources are widened, the same conversion the kernels apply on the fly), zero-padded to whole tiles,
 * tile (i, j) = rows 128 i .., cols 128 j .. stored at (i * ceil(cols / 128) + j) * 32768 bytes; inside a tile,
 * element (k, n) is the half at  k * 128 + (((n / 32) ^ (k % 4)) * 32) + n % 32.
 * fsvd_tiled_bytes gives the buffer size (0 if rows or cols is not positive, cols % 8 != 0, or the image would
 * reach 2 GiB); fsvd_pack_tiled converts a contiguous row-major [rows, cols] matrix (F16 or BF16).  With tile images
 * the kernels do the same arithmetic as with row-major weights (outputs agree up to the last bit).  Matrices accepted as
 * FSVD_TILED: U and V of every whole-matrix factor (q, k, v, o, w1, w2) and U of per-head factors; V of a per-head
 * factor must be row-major.  Matrices that are read by one launch must be given alike, else FSVD_ERR_UNSUPPORTED:
 * U of q, k, v; V of q, k, v; V of w1 and U of w2.  The FFN core copies tile images into on-chip memory with direct
 * loads; the projections and the attention rebuild read them in place of the row-major matrix (no conversion,
 * contiguous requests).
 */
size_t fsvd_tiled_bytes(int32_t rows, int32_t cols);
fsvd_status fsvd_pack_tiled(int32_t rows, int32_t cols, const void *src, fsvd_dtype src_dtype, void *dst,
                            void *hip_stream);

/* Alg. 1 Part II on rank-space inputs: Pq [B*M, q->rank], Pk, Pv (FM) and the V / bias members of
 * q, k, v (their U members are ignored) -> context [B*M, D] (FM, heads concatenated). */
fsvd_status fsvd_attention_core(const fsvd_desc *desc, const void *Pq, const void *Pk, const void *Pv,
                                const fsvd_factor *q, const fsvd_factor *k, const fsvd_factor *v,
                                void *context, void *hip_stream);
/* The same with per-head factors (see fsvd_attention_heads): Pq, Pk, Pv are [B*M, H * rank] (FM). */
fsvd_status fsvd_attention_heads_core(const fsvd_desc *desc, const void *Pq, const void *Pk, const void *Pv,
                                      const fsvd_factor *q, const fsvd_factor *k, const fsvd_factor *v,
                                      void *context, void *hip_stream);

/* The on-chip loops of Alg. 2: P1 [B*M, w1->rank] (FM), V / bias of w1 and U of w2 -> Z [B*M, w2->rank]
 * (FM) with Z = phi(P1 V_1 + b_1) U_2.  When few tokens or large ranks would leave compute units idle the sum over
 * D_ff is split across workgroups and their fp32 partial sums are added in a fixed order by a second launch; the
 * partial sums live in `workspace` (256-byte aligned device memory of at least fsvd_ffn_core_workspace() bytes, which
 * is 0 when no split is used and never more than B*M*F bytes; NULL is accepted when it is 0). */
size_t fsvd_ffn_core_workspace(const fsvd_desc *desc, int32_t r_1, int32_t r_2);
fsvd_status fsvd_ffn_core(const fsvd_desc *desc, const void *P1, const fsvd_factor *w1, const fsvd_factor *w2,
                          void *Z, void *workspace, size_t workspace_bytes, void *hip_stream);

/* ------------------------------------------------------------------------------------------
 * Decoding step against a rank-space KV cache (appendix on decoder models, "Prefill" / "Decoding Phase": the
 * cache holds P_k = X U_k and P_v = X U_v, 2 t r scalars per sequence instead of 2 t D, and a step attends one new
 * query to the cached rows).  Whole-matrix factors; desc->M is the cache capacity t_max (tokens per sequence),
 * desc->causal, key_len, F, act and norm are ignored.  Limits: r_k % 64 == 0, r_v % 32 == 0, both <= 1024, H <= 32,
 * V of k and v row-major; FSVD_ERR_UNSUPPORTED otherwise.
 *
 * The two caches are device buffers owned by the caller, in layouts private to the library (so that a cached block is
 * a matrix-core operand as it lies in memory); fsvd_decode_kcache_bytes / fsvd_decode_vcache_bytes give their sizes
 * (0 for invalid arguments).  A new cache must be ZERO-FILLED by the caller: positions never written are masked, but
 * they must hold finite values.  Sequence b of a cache starts at b * (bytes / B).
 *
 * fsvd_decode_cache_write stores rows P_new [B, n_new, r] (fp16, row-major) at positions t_start[b] .. t_start[b] +
 * n_new - 1 of sequence b (t_start: device int32[B]); which = 0 writes the K cache, 1 the V cache; rows that would fall
 * at or beyond t_max are dropped.  It serves to load the result of a prefill; fsvd_decode_attention appends the new
 * token's rows itself.
 *
 * fsvd_decode_attention, for every sequence b with t_len[b] cached tokens (device int32[B], 0 <= t_len[b] < t_max):
 *   p_a = x_new[b] U_a for a in {q, k, v};  p_k, p_v are written to position t_len[b] of the caches;
 *   per head h: scores_j = (p_q V_q + b_q)_h . (P_k[j] V_k + b_k)_h * softmax_scale for j = 0 .. t_len[b],
 *   evaluated as P_k[j] . (V_k[:, h] q_h) (the b_k term is the same for every key and cancels in the softmax);
 *   context_h = (sum_j a_j P_v[j]) V_v[:, h] + b_v[h];   out[b] = (context U_o) V_o + b_o.
 * x_new [B, D] in io_dtype -> out [B, D] in out_dtype.  The caller advances t_len after the call.  K and V are never
 * rebuilt; per sequence the step reads (t_len + 1) (r_k + r_v) 2 bytes of cache once for all heads.
 * ------------------------------------------------------------------------------------------ */
size_t fsvd_decode_kcache_bytes(int32_t B, int32_t t_max, int32_t r_k);
size_t fsvd_decode_vcache_bytes(int32_t B, int32_t t_max, int32_t r_v);
fsvd_status fsvd_decode_cache_write(int32_t B, int32_t t_max, int32_t r, int32_t n_new, const int32_t *t_start,
                                    const void *P_new, int32_t which, void *cache, void *hip_stream);
size_t fsvd_decode_attention_workspace(const fsvd_desc *desc, int32_t r_q, int32_t r_k, int32_t r_v, int32_t r_o);
fsvd_status fsvd_decode_attention(const fsvd_desc *desc, const void *x_new, const fsvd_factor *q, const fsvd_factor *k,
                                  const fsvd_factor *v, const fsvd_factor *o, void *kcache, void *vcache,
                                  const int32_t *t_len, void *out, void *workspace, size_t workspace_bytes,
                                  void *hip_stream);
/* Building block: the pass over the cache alone.  W: the absorbed queries, per sequence the fragment-major layout of
 * a [32, r_k] fp16 matrix whose row h < H is softmax_scale * log2(e) * V_k[:, head h] q_h (rows >= H are ignored);
 * n_keys: device int32[B], the number of valid cached keys per sequence (1 .. t_max);
 * u_out [B, H, r_v] fp32 = sum_j a_j P_v[j] per head.  The keys of a sequence are split over several workgroups whose
 * partial results (fp16 sums, fp32 softmax statistics) pass through `workspace` and are merged in a fixed order. */
size_t fsvd_decode_core_workspace(const fsvd_desc *desc, int32_t r_k, int32_t r_v);
fsvd_status fsvd_decode_attention_core(const fsvd_desc *desc, int32_t r_k, int32_t r_v, const void *W,
                                       const void *kcache, const void *vcache, const int32_t *n_keys, void *u_out,
                                       void *workspace, size_t workspace_bytes, void *hip_stream);

/* Y[T, D] = gamma (X - mean) / sqrt(var + eps) + beta per row; X in x_dtype, gamma / beta in p_dtype,
 * Y in y_dtype (any of F16, BF16, F32).  D <= 8192, D % 8 == 0. */
fsvd_status fsvd_layernorm(int32_t T, int32_t D, const void *X, fsvd_dtype x_dtype, const void *gamma,
                           const void *beta, fsvd_dtype p_dtype, float eps, void *Y, fsvd_dtype y_dtype,
                           void *hip_stream);

/* Measurement aid (no part of the method): launches `workgroups` workgroups of four wavefronts that each execute
 * iters x 4 v_mfma_f32_32x32x16_f16 instructions (32768 FLOP each) on register-resident operands, nothing read from
 * memory; total FLOP = workgroups * 4 * iters * 4 * 32768.  The benchmark times it to state the matrix-core rate the
 * part sustains under load beside the published peak.  out: device float[workgroups * 256], overwritten.
 * workgroups in [1, 65536], iters in [1, 2^20]. */
fsvd_status fsvd_mfma_probe(int32_t workgroups, int32_t iters, void *out, void *hip_stream);

/* Measurement aid (no part of the method): the rate at which a compute unit can be fed from the L2 with the
 * direct-to-LDS loads the fused kernels use.  Launches `workgroups` workgroups of eight wavefronts; each copies `steps`
 * steps of 32 KiB straight into LDS (four 1 KiB loads per wavefront and step, two steps in flight, no barrier), all
 * workgroups of one XCD walking the same region of `region_bytes` bytes of `src` (eight regions, one per XCD, so the
 * data comes out of that XCD's L2 after the first touch); with_work != 0 adds twelve 16-byte LDS reads and eight
 * MFMAs per wavefront and step, the operand traffic and matrix-core load of a stage of the fused FFN core.  Bytes
 * moved = workgroups * steps * 32768.  src: device buffer of 8 * region_bytes bytes; region_bytes a multiple of 32768,
 * at most 2^30; out: device float[workgroups * 512], overwritten.  workgroups in [1, 65536], steps in [1, 2^20]. */
fsvd_status fsvd_dma_probe(int32_t workgroups, int32_t steps, int32_t with_work, const void *src, size_t region_bytes,
                           void *out, void *hip_stream);

/* Static, NUL-terminated description of a status code. */
const char *fsvd_status_string(fsvd_status status);

/* Library version, major * 10000 + minor * 100 + patch. */
int32_t fsvd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FSVD_H */
