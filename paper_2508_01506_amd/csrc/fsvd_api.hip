// C-ABI entry points: argument validation, workspace carving and the launch sequence of one layer.
// Everything here is host code; validation and the workspace functions touch no device.
#include "../../include/fsvd.h"
#include "fsvd_common.h"
#include "fsvd_kernels.h"

#include <mutex>

using namespace fsvd;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t n) { return (n + kAlign - 1) / kAlign * kAlign; }
inline bool dtype_ok16(int d) { return d == FSVD_F16 || d == FSVD_BF16; }
inline bool dtype_ok(int d) { return d == FSVD_F16 || d == FSVD_BF16 || d == FSVD_F32; }
inline size_t smax(size_t a, size_t b) { return a > b ? a : b; }
// every tensor is read and written with 16-byte vector accesses
inline bool mis16(const void* p) { return p && ((uintptr_t)p & 15) != 0; }

fsvd_status check_desc(const fsvd_desc* d, bool need_ffn) {
  if (!d) return FSVD_ERR_INVALID_ARG;
  if (d->B <= 0 || d->M <= 0 || d->D <= 0 || d->H <= 0) return FSVD_ERR_INVALID_ARG;
  if (need_ffn && d->F <= 0) return FSVD_ERR_INVALID_ARG;
  if (!dtype_ok16(d->io_dtype) || !dtype_ok(d->out_dtype)) return FSVD_ERR_INVALID_ARG;
  if (d->act < FSVD_ACT_GELU_ERF || d->act > FSVD_ACT_RELU) return FSVD_ERR_INVALID_ARG;
  if (d->norm < FSVD_NORM_NONE || d->norm > FSVD_NORM_PRE_LN) return FSVD_ERR_INVALID_ARG;
  if (!(d->softmax_scale >= 0.f) || !(d->ln_eps >= 0.f)) return FSVD_ERR_INVALID_ARG;
  if (d->D % d->H != 0) return FSVD_ERR_INVALID_ARG;
  const int dh = d->D / d->H;
  if (dh != 64 && dh != 128) return FSVD_ERR_UNSUPPORTED;
  if (d->D % 16 != 0 || d->D > 8192) return FSVD_ERR_UNSUPPORTED;
  if (need_ffn && d->F % 16 != 0) return FSVD_ERR_UNSUPPORTED;
  const long long widest = need_ffn && d->F > d->D ? d->F : d->D;
  if ((long long)d->B * d->M * widest >= (1LL << 29)) return FSVD_ERR_UNSUPPORTED;   // every tensor < 2 GiB
  return FSVD_OK;
}

fsvd_status check_rank(int r) {
  if (r <= 0) return FSVD_ERR_INVALID_ARG;
  if (r % 16 != 0) return FSVD_ERR_UNSUPPORTED;
  return FSVD_OK;
}

// pointers are only required when a computation is about to run (need_ptrs)
// tiled_ok: bit 0 = U may be given as tile images, bit 1 = V may be
fsvd_status check_factor(const fsvd_factor* f, int in_dim, int out_dim, bool need_u, bool need_v, int tiled_ok = 0) {
  if (!f) return FSVD_ERR_INVALID_ARG;
  for (const int l : {f->u_layout, f->v_layout})
    if (l != FSVD_ROW_MAJOR && l != FSVD_TILED) return FSVD_ERR_INVALID_ARG;
  if (f->u_layout == FSVD_TILED && !(tiled_ok & 1)) return FSVD_ERR_UNSUPPORTED;
  if (f->v_layout == FSVD_TILED && !(tiled_ok & 2)) return FSVD_ERR_UNSUPPORTED;
  if (f->in_dim != in_dim || f->out_dim != out_dim) return FSVD_ERR_INVALID_ARG;
  fsvd_status s = check_rank(f->rank);
  if (s != FSVD_OK) return s;
  const long long widest = in_dim > out_dim ? in_dim : out_dim;
  if ((long long)f->rank * widest >= (1LL << 29)) return FSVD_ERR_UNSUPPORTED;   // each factor < 1 GiB
  if (need_u && !f->U) return FSVD_ERR_INVALID_ARG;
  if (need_v && !f->V) return FSVD_ERR_INVALID_ARG;
  if (mis16(f->U) || mis16(f->V) || mis16(f->bias)) return FSVD_ERR_INVALID_ARG;
  return FSVD_OK;
}

#define FSVD_TRY(expr) do { fsvd_status _s = (expr); if (_s != FSVD_OK) return _s; } while (0)
#define FSVD_HIP(expr) do { if ((expr) != hipSuccess) return FSVD_ERR_DEVICE; } while (0)

fsvd_status check_attn(const fsvd_desc* d, const fsvd_factor* q, const fsvd_factor* k, const fsvd_factor* v,
                       const fsvd_factor* o, bool ptrs) {
  FSVD_TRY(check_desc(d, false));
  FSVD_TRY(check_factor(q, d->D, d->D, ptrs, ptrs, 3));
  FSVD_TRY(check_factor(k, d->D, d->D, ptrs, ptrs, 3));
  FSVD_TRY(check_factor(v, d->D, d->D, ptrs, ptrs, 3));
  FSVD_TRY(check_factor(o, d->D, d->D, ptrs, ptrs, 3));
  // q, k and v share one projection launch and one rebuild launch: one weight path per launch
  if (q->u_layout != k->u_layout || q->u_layout != v->u_layout) return FSVD_ERR_UNSUPPORTED;
  if (q->v_layout != k->v_layout || q->v_layout != v->v_layout) return FSVD_ERR_UNSUPPORTED;
  return FSVD_OK;
}
// number of groups of a grouped factor: the `groups` member, 0 meaning one group per head
inline int groups_of(const fsvd_desc* d, const fsvd_factor* f) { return f->groups > 0 ? f->groups : d->H; }
// grouped (per-head) factors of q, k, v: in_dim = out_dim = D, `rank` is the rank of ONE group
fsvd_status check_attn_heads(const fsvd_desc* d, const fsvd_factor* q, const fsvd_factor* k, const fsvd_factor* v,
                             const fsvd_factor* o, bool ptrs) {
  FSVD_TRY(check_desc(d, false));
  for (const fsvd_factor* f : {q, k, v}) {
    FSVD_TRY(check_factor(f, d->D, d->D, ptrs, ptrs, 1));      // U [D, G r] feeds a plain projection; V stays row-major
    if (f->groups < 0 || d->H % groups_of(d, f) != 0) return FSVD_ERR_INVALID_ARG;
    if (f->groups != q->groups) return FSVD_ERR_UNSUPPORTED;
    if ((long long)f->rank * groups_of(d, f) * d->D >= (1LL << 29)) return FSVD_ERR_UNSUPPORTED;
  }
  if (q->u_layout != k->u_layout || q->u_layout != v->u_layout) return FSVD_ERR_UNSUPPORTED;
  FSVD_TRY(check_factor(o, d->D, d->D, ptrs, ptrs, 3));
  return FSVD_OK;
}
fsvd_status check_ffn(const fsvd_desc* d, const fsvd_factor* w1, const fsvd_factor* w2, bool ptrs) {
  FSVD_TRY(check_desc(d, true));
  FSVD_TRY(check_factor(w1, d->D, d->F, ptrs, ptrs, 3));
  FSVD_TRY(check_factor(w2, d->F, d->D, ptrs, ptrs, 3));
  if (w1->v_layout != w2->u_layout) return FSVD_ERR_UNSUPPORTED;   // the fused core reads both streams the same way
  return FSVD_OK;
}
fsvd_status check_ws(const void* ws, size_t have, size_t need) {
  if (!ws || ((uintptr_t)ws % kAlign) != 0 || have < need) return FSVD_ERR_WORKSPACE;
  return FSVD_OK;
}

// ---- workspace plans (bytes).  Every intermediate that feeds a matrix-core contraction is fp16 in the
// fragment-major layout (fm_bytes pads tokens to 32 and the contraction axis to 64); the residual stream is fp32.
struct AttnPlan { size_t c, p, pq, pk, pv, to, total; };   // C (also the packed X); P_q | P_k | P_v; T_o aliases P
AttnPlan plan_attn(size_t T, size_t D, size_t rq, size_t rk, size_t rv, size_t ro) {
  AttnPlan pl;
  pl.c = 0;
  pl.p = align_up(fm_bytes(T, D));
  pl.pq = pl.p;
  pl.pk = pl.pq + align_up(fm_bytes(T, rq));
  pl.pv = pl.pk + align_up(fm_bytes(T, rk));
  const size_t p_end = pl.pv + align_up(fm_bytes(T, rv));
  pl.to = pl.p;
  pl.total = smax(p_end, pl.to + align_up(fm_bytes(T, ro)));
  return pl;
}
// The size queries do not know the weight layout: room for the larger of the two kernels' partial sums.
size_t ffn_core_partial_bytes(int T, int r1, int r2, int F) {
  return smax(ffn_core_plan(T, r1, r2, F, false).partial_bytes, ffn_core_plan(T, r1, r2, F, true).partial_bytes);
}
struct FfnPlan { size_t p1, z, part, total; };   // P1 | Z | fp32 partial sums of Z (only when the core splits F)
FfnPlan plan_ffn(size_t T, size_t r1, size_t r2, size_t F) {
  FfnPlan pl;
  pl.p1 = 0;
  pl.z = align_up(fm_bytes(T, r1));
  pl.part = pl.z + align_up(fm_bytes(T, r2));
  pl.total = pl.part + align_up(ffn_core_partial_bytes((int)T, (int)r1, (int)r2, (int)F));
  return pl;
}

// LayerNorm to be applied to the block's output (after the residual add).  When the block's last projection can be
// fused with it (prepacked V, supported width) the block writes the normalised rows and sets `done`; otherwise the
// block writes its plain output and the caller normalises it.
struct LnFuse {
  const void* gamma; const void* beta; float eps;
  void* y_row; int y_dt;      // normalised rows, row-major (or nullptr)
  void* y_fm;                 // fragment-major fp16 copy (or nullptr)
  bool done;
};
// The fused projection + residual + LayerNorm kernel gives every workgroup all D output columns of 32 or 64 tokens, so
// each workgroup re-reads the whole [rank, D] matrix from the last-level cache: it wins over the GEMM followed by the
// LayerNorm kernel (one more round trip of [T, D] through HBM, one more launch) while that matrix is moderate; measured
// from 256 tokens up and for rank x D up to 768 Ki.
bool ln_fusable(const fsvd_desc* d, const fsvd_factor* last) {
  return last->v_layout == FSVD_TILED && linear_ln_supported(d->D) && d->B * d->M >= 256 &&
         (long long)last->rank * d->D <= 768 * 1024 && linear_ln_fits((long long)d->B * d->M, d->D);
}

float resolve_scale(const fsvd_desc* d) {
  return d->softmax_scale > 0.f ? d->softmax_scale : 1.0f / sqrtf((float)(d->D / d->H));
}

// Attention block.  `x_fm`: the block input, fragment-major fp16 [T, D] (it may live in c_buf: the context
// overwrites it only after the rank projection has consumed it).  c_buf: FM [T, D]; rank_buf: P_q | P_k | P_v, later T_o.
// The last GEMM writes `out` row-major in c_dt (+ residual) or, when out_fm is set, fragment-major fp16.
fsvd_status run_attention(const fsvd_desc* d, const void* x_fm, const fsvd_factor* q, const fsvd_factor* k,
                          const fsvd_factor* v, const fsvd_factor* o, const void* residual, int r_dt, void* out,
                          int c_dt, bool out_fm, char* c_buf, char* rank_buf, hipStream_t s, bool per_head = false,
                          LnFuse* lnf = nullptr) {
  const int T = d->B * d->M, D = d->D;
  // per-head factors: U [D, H r] is one projection matrix with H r columns, head h's rank-space activations are
  // columns h r .. of P; V [H, r, d_h] is read per head by the attention core
  const int G = per_head ? groups_of(d, q) : 1;
  const int hq = G * q->rank, hk = G * k->rank, hv = G * v->rank;
  const AttnPlan pl = plan_attn(T, D, hq, hk, hv, o->rank);
  char* Pq = rank_buf;
  char* Pk = rank_buf + (pl.pk - pl.p);
  char* Pv = rank_buf + (pl.pv - pl.p);
  char* To = rank_buf;   // P is dead once the context is complete

  LinearArgs h1{};
  h1.A = x_fm; h1.a_layout = LAYOUT_FM; h1.lda = D; h1.a_dt = DT_F16; h1.T = T; h1.K = D; h1.w_dt = d->io_dtype;
  h1.w_tiled = q->u_layout == FSVD_TILED;
  h1.c_layout = LAYOUT_FM; h1.c_dt = DT_F16; h1.R = nullptr; h1.ngroups = 3;
  h1.g[0] = {q->U, nullptr, Pq, hq, hq, 0};
  h1.g[1] = {k->U, nullptr, Pk, hk, hk, 0};
  h1.g[2] = {v->U, nullptr, Pv, hv, hv, 0};
  FSVD_HIP(launch_linear(h1, s));

  AttnCoreArgs ca{};
  ca.Pq = Pq; ca.Pk = Pk; ca.Pv = Pv;
  ca.rq = q->rank; ca.rk = k->rank; ca.rv = v->rank; ca.per_head = per_head ? d->H / G : 0;
  ca.Vq = q->V; ca.Vk = k->V; ca.Vv = v->V;
  ca.bq = q->bias; ca.bk = k->bias; ca.bv = v->bias;
  ca.w_dt = d->io_dtype; ca.tiled = q->v_layout == FSVD_TILED;
  ca.B = d->B; ca.M = d->M; ca.D = D; ca.H = d->H;
  ca.causal = d->causal; ca.key_len = d->key_len; ca.scale = resolve_scale(d);
  ca.C = c_buf;
  FSVD_HIP(launch_attn_core(ca, s));

  LinearArgs h3a{};
  h3a.A = c_buf; h3a.a_layout = LAYOUT_FM; h3a.lda = D; h3a.a_dt = DT_F16; h3a.T = T; h3a.K = D; h3a.w_dt = d->io_dtype;
  h3a.w_tiled = o->u_layout == FSVD_TILED;
  h3a.c_layout = LAYOUT_FM; h3a.c_dt = DT_F16; h3a.ngroups = 1;
  h3a.g[0] = {o->U, nullptr, To, o->rank, o->rank, 0};
  FSVD_HIP(launch_linear(h3a, s));

  if (lnf && ln_fusable(d, o)) {
    LinearLnArgs f{};
    f.A = To; f.T = T; f.K = o->rank; f.D = D; f.W = o->V; f.bias = o->bias; f.w_dt = d->io_dtype;
    f.R = residual; f.r_dt = r_dt; f.gamma = lnf->gamma; f.beta = lnf->beta; f.p_dt = d->io_dtype; f.eps = lnf->eps;
    f.Yrow = lnf->y_row; f.yrow_dt = lnf->y_dt; f.Yfm = lnf->y_fm;
    FSVD_HIP(launch_linear_ln(f, s));
    lnf->done = true;
    return FSVD_OK;
  }
  LinearArgs h3b{};
  h3b.A = To; h3b.a_layout = LAYOUT_FM; h3b.lda = o->rank; h3b.a_dt = DT_F16; h3b.T = T; h3b.K = o->rank;
  h3b.w_dt = d->io_dtype; h3b.w_tiled = o->v_layout == FSVD_TILED; h3b.c_layout = out_fm ? LAYOUT_FM : LAYOUT_ROW; h3b.c_dt = c_dt;
  h3b.R = residual; h3b.ldr = D; h3b.r_dt = r_dt; h3b.ngroups = 1;
  h3b.g[0] = {o->V, o->bias, out, D, D, D};
  FSVD_HIP(launch_linear(h3b, s));
  return FSVD_OK;
}

// FFN block on `A_in` (fragment-major fp16, or row-major in a_dt) -> row-major `out` in c_dt (+ residual).
fsvd_status run_ffn(const fsvd_desc* d, const void* A_in, int a_layout, int a_dt, const fsvd_factor* w1,
                    const fsvd_factor* w2, const void* residual, int r_dt, void* out, int c_dt, char* scratch,
                    hipStream_t s, LnFuse* lnf = nullptr) {
  const int T = d->B * d->M, D = d->D;
  const FfnPlan pl = plan_ffn(T, w1->rank, w2->rank, d->F);
  char* P1 = scratch + pl.p1;
  char* Z = scratch + pl.z;

  LinearArgs h5{};
  h5.A = A_in; h5.a_layout = a_layout; h5.lda = D; h5.a_dt = a_dt; h5.T = T; h5.K = D; h5.w_dt = d->io_dtype;
  h5.w_tiled = w1->u_layout == FSVD_TILED;
  h5.c_layout = LAYOUT_FM; h5.c_dt = DT_F16; h5.ngroups = 1;
  h5.g[0] = {w1->U, nullptr, P1, w1->rank, w1->rank, 0};
  FSVD_HIP(launch_linear(h5, s));

  FfnCoreArgs fa{};
  fa.P1 = P1; fa.r1 = w1->rank; fa.V1 = w1->V; fa.b1 = w1->bias; fa.U2 = w2->U; fa.r2 = w2->rank;
  fa.w_dt = d->io_dtype; fa.tiled = w1->v_layout == FSVD_TILED; fa.T = T; fa.F = d->F; fa.act = d->act; fa.Z = Z;
  fa.Zpart = (float*)(scratch + pl.part);
  FSVD_HIP(launch_ffn_core(fa, s));

  if (lnf && ln_fusable(d, w2)) {
    LinearLnArgs f{};
    f.A = Z; f.T = T; f.K = w2->rank; f.D = D; f.W = w2->V; f.bias = w2->bias; f.w_dt = d->io_dtype;
    f.R = residual; f.r_dt = r_dt; f.gamma = lnf->gamma; f.beta = lnf->beta; f.p_dt = d->io_dtype; f.eps = lnf->eps;
    f.Yrow = lnf->y_row; f.yrow_dt = lnf->y_dt; f.Yfm = lnf->y_fm;
    FSVD_HIP(launch_linear_ln(f, s));
    lnf->done = true;
    return FSVD_OK;
  }
  LinearArgs h7{};
  h7.A = Z; h7.a_layout = LAYOUT_FM; h7.lda = w2->rank; h7.a_dt = DT_F16; h7.T = T; h7.K = w2->rank; h7.w_dt = d->io_dtype;
  h7.w_tiled = w2->v_layout == FSVD_TILED;
  h7.c_layout = LAYOUT_ROW; h7.c_dt = c_dt; h7.R = residual; h7.ldr = D; h7.r_dt = r_dt; h7.ngroups = 1;
  h7.g[0] = {w2->V, w2->bias, out, D, D, D};
  FSVD_HIP(launch_linear(h7, s));
  return FSVD_OK;
}

// layer workspace: [residual stream: fp32 [T, D] row-major (absent for NORM_NONE)] [FM [T, D]: packed input / context /
// normalised copy] [rank scratch: max(P_q|P_k|P_v, T_o, P1 + Z)]
struct LayerPlan { size_t stream, c, rank, total; };
LayerPlan plan_layer(const fsvd_desc* d, size_t rq, size_t rk, size_t rv, size_t ro, size_t r1, size_t r2) {
  const size_t T = (size_t)d->B * d->M, D = d->D;
  LayerPlan pl;
  pl.stream = 0;
  pl.c = d->norm == FSVD_NORM_NONE ? 0 : align_up(T * D * 4);
  pl.rank = pl.c + align_up(fm_bytes(T, D));
  const AttnPlan ap = plan_attn(T, D, rq, rk, rv, ro);
  pl.total = pl.rank + smax(ap.total - ap.p, plan_ffn(T, r1, r2, d->F).total);
  return pl;
}

}  // namespace

extern "C" {

const char* fsvd_status_string(fsvd_status s) {
  switch (s) {
    case FSVD_OK: return "ok";
    case FSVD_ERR_INVALID_ARG: return "invalid argument";
    case FSVD_ERR_UNSUPPORTED: return "unsupported configuration";
    case FSVD_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case FSVD_ERR_DEVICE: return "device launch failed";
  }
  return "unknown status";
}

int32_t fsvd_version(void) { return 100; }

size_t fsvd_attention_workspace(const fsvd_desc* d, int32_t rq, int32_t rk, int32_t rv, int32_t ro) {
  if (check_desc(d, false) != FSVD_OK) return 0;
  if (check_rank(rq) || check_rank(rk) || check_rank(rv) || check_rank(ro)) return 0;
  return plan_attn((size_t)d->B * d->M, d->D, rq, rk, rv, ro).total;
}
size_t fsvd_ffn_workspace(const fsvd_desc* d, int32_t r1, int32_t r2) {
  if (check_desc(d, true) != FSVD_OK) return 0;
  if (check_rank(r1) || check_rank(r2)) return 0;
  return plan_ffn((size_t)d->B * d->M, r1, r2, d->F).total;
}
size_t fsvd_layer_workspace(const fsvd_desc* d, int32_t rq, int32_t rk, int32_t rv, int32_t ro, int32_t r1, int32_t r2) {
  if (check_desc(d, true) != FSVD_OK) return 0;
  if (check_rank(rq) || check_rank(rk) || check_rank(rv) || check_rank(ro) || check_rank(r1) || check_rank(r2)) return 0;
  return plan_layer(d, rq, rk, rv, ro, r1, r2).total;
}

fsvd_status fsvd_attention_check(const fsvd_desc* d, const fsvd_factor* q, const fsvd_factor* k, const fsvd_factor* v,
                                 const fsvd_factor* o) {
  return check_attn(d, q, k, v, o, false);
}
fsvd_status fsvd_ffn_check(const fsvd_desc* d, const fsvd_factor* w1, const fsvd_factor* w2) {
  return check_ffn(d, w1, w2, false);
}

fsvd_status fsvd_attention(const fsvd_desc* d, const void* X, const fsvd_factor* q, const fsvd_factor* k,
                           const fsvd_factor* v, const fsvd_factor* o, void* out, void* ws, size_t ws_bytes, void* stream) {
  FSVD_TRY(check_attn(d, q, k, v, o, true));
  if (!X || !out || mis16(X) || mis16(out)) return FSVD_ERR_INVALID_ARG;
  const int T = d->B * d->M;
  const AttnPlan pl = plan_attn(T, d->D, q->rank, k->rank, v->rank, o->rank);
  FSVD_TRY(check_ws(ws, ws_bytes, pl.total));
  hipStream_t s = (hipStream_t)stream;
  char* w = (char*)ws;
  FSVD_HIP(launch_pack_fm(X, d->io_dtype, T, d->D, w + pl.c, s));
  return run_attention(d, w + pl.c, q, k, v, o, nullptr, 0, out, d->out_dtype, false, w + pl.c, w + pl.p, s);
}

size_t fsvd_attention_groups_workspace(const fsvd_desc* d, int32_t groups, int32_t rq, int32_t rk, int32_t rv, int32_t ro) {
  if (check_desc(d, false) != FSVD_OK) return 0;
  if (check_rank(rq) || check_rank(rk) || check_rank(rv) || check_rank(ro)) return 0;
  const size_t G = groups > 0 ? groups : d->H;
  if (groups < 0 || d->H % G != 0) return 0;
  return plan_attn((size_t)d->B * d->M, d->D, G * rq, G * rk, G * rv, ro).total;
}
size_t fsvd_attention_heads_workspace(const fsvd_desc* d, int32_t rq, int32_t rk, int32_t rv, int32_t ro) {
  return fsvd_attention_groups_workspace(d, 0, rq, rk, rv, ro);
}

fsvd_status fsvd_attention_heads(const fsvd_desc* d, const void* X, const fsvd_factor* q, const fsvd_factor* k,
                                 const fsvd_factor* v, const fsvd_factor* o, void* out, void* ws, size_t ws_bytes,
                                 void* stream) {
  FSVD_TRY(check_attn_heads(d, q, k, v, o, true));
  if (!X || !out || mis16(X) || mis16(out)) return FSVD_ERR_INVALID_ARG;
  const int T = d->B * d->M;
  const size_t G = groups_of(d, q);
  const AttnPlan pl = plan_attn(T, d->D, G * q->rank, G * k->rank, G * v->rank, o->rank);
  FSVD_TRY(check_ws(ws, ws_bytes, pl.total));
  hipStream_t s = (hipStream_t)stream;
  char* w = (char*)ws;
  FSVD_HIP(launch_pack_fm(X, d->io_dtype, T, d->D, w + pl.c, s));
  return run_attention(d, w + pl.c, q, k, v, o, nullptr, 0, out, d->out_dtype, false, w + pl.c, w + pl.p, s, true);
}

fsvd_status fsvd_ffn(const fsvd_desc* d, const void* X, const fsvd_factor* w1, const fsvd_factor* w2, void* out,
                     void* ws, size_t ws_bytes, void* stream) {
  FSVD_TRY(check_ffn(d, w1, w2, true));
  if (!X || !out || mis16(X) || mis16(out)) return FSVD_ERR_INVALID_ARG;
  FSVD_TRY(check_ws(ws, ws_bytes, plan_ffn((size_t)d->B * d->M, w1->rank, w2->rank, d->F).total));
  return run_ffn(d, X, LAYOUT_ROW, d->io_dtype, w1, w2, nullptr, 0, out, d->out_dtype, (char*)ws, (hipStream_t)stream);
}

}  // extern "C"

// ------------------------------------------------------------------ fsvd_ffn without a caller workspace
// The scratch of fsvd_ffn_static: part of the device image, one copy per GPU.  In host code the array's name is only a
// handle for the runtime's symbol lookup, never an address a kernel may use: scratch_of_current_device() asks the
// runtime once per device for the array's address on that device, and only that address is handed to kernels.
namespace {
static __device__ __align__(256) unsigned char scratch[FSVD_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];      // per device: address of `scratch` on that device (nullptr = not looked up yet)
std::mutex g_scratch_mu;

fsvd_status scratch_of_current_device(char** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return FSVD_ERR_DEVICE;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return FSVD_ERR_DEVICE;
    g_scratch_ptr[dev] = p;
  }
  *out = (char*)g_scratch_ptr[dev];
  return FSVD_OK;
}
}  // namespace

extern "C" {

fsvd_status fsvd_ffn_static(const fsvd_desc* d, const void* X, const fsvd_factor* w1, const fsvd_factor* w2, void* out,
                            void* stream) {
  FSVD_TRY(check_ffn(d, w1, w2, true));
  if (!X || !out || mis16(X) || mis16(out)) return FSVD_ERR_INVALID_ARG;
  if (plan_ffn((size_t)d->B * d->M, w1->rank, w2->rank, d->F).total > FSVD_STATIC_SCRATCH_BYTES) return FSVD_ERR_WORKSPACE;
  char* ws = nullptr;
  FSVD_TRY(scratch_of_current_device(&ws));
  return run_ffn(d, X, LAYOUT_ROW, d->io_dtype, w1, w2, nullptr, 0, out, d->out_dtype, ws, (hipStream_t)stream);
}

fsvd_status fsvd_ffn_v2(const fsvd_desc* d, const void* X, const fsvd_factor* w1, const fsvd_factor* w2, void* out,
                        void* stream) {
  FSVD_TRY(check_ffn(d, w1, w2, true));
  if (!X || !out || mis16(X) || mis16(out)) return FSVD_ERR_INVALID_ARG;
  for (const fsvd_factor* f : {w1, w2})
    if (f->u_layout != FSVD_TILED || f->v_layout != FSVD_TILED) return FSVD_ERR_UNSUPPORTED;
  if (!ffn_v2_supported(d->D, d->F, w1->rank, w2->rank)) return FSVD_ERR_UNSUPPORTED;
  FfnV2Args a{};
  a.X = X; a.x_dt = d->io_dtype;
  a.U1 = w1->U; a.V1 = w1->V; a.U2 = w2->U; a.V2 = w2->V; a.b1 = w1->bias; a.b2 = w2->bias; a.w_dt = d->io_dtype;
  a.T = d->B * d->M; a.D = d->D; a.F = d->F; a.r1 = w1->rank; a.r2 = w2->rank; a.act = d->act;
  a.out = out; a.out_dt = d->out_dtype;
  FSVD_HIP(launch_ffn_v2(a, (hipStream_t)stream));
  return FSVD_OK;
}

}  // extern "C"

namespace {
fsvd_status layer_impl(const fsvd_desc* d, const void* X, const fsvd_factor* q, const fsvd_factor* k,
                       const fsvd_factor* v, const fsvd_factor* o, const void* g1, const void* b1,
                       const fsvd_factor* w1, const fsvd_factor* w2, const void* g2, const void* b2, void* out,
                       void* ws, size_t ws_bytes, void* stream, bool per_head) {
  FSVD_TRY(per_head ? check_attn_heads(d, q, k, v, o, true) : check_attn(d, q, k, v, o, true));
  FSVD_TRY(check_ffn(d, w1, w2, true));
  if (!X || !out || mis16(X) || mis16(out)) return FSVD_ERR_INVALID_ARG;
  if (d->norm != FSVD_NORM_NONE && (!g1 || !b1 || !g2 || !b2)) return FSVD_ERR_INVALID_ARG;
  if (mis16(g1) || mis16(b1) || mis16(g2) || mis16(b2)) return FSVD_ERR_INVALID_ARG;
  const size_t hm = per_head ? (size_t)groups_of(d, q) : 1;     // grouped factors: G * rank columns of P per projection
  const LayerPlan pl = plan_layer(d, hm * q->rank, hm * k->rank, hm * v->rank, o->rank, w1->rank, w2->rank);
  FSVD_TRY(check_ws(ws, ws_bytes, pl.total));
  hipStream_t s = (hipStream_t)stream;
  char* w = (char*)ws;
  char* stream_buf = w + pl.stream;
  char* c_buf = w + pl.c;
  char* rank_buf = w + pl.rank;
  const int T = d->B * d->M, D = d->D;
  const int io = d->io_dtype;

  auto ln = [&](const void* x, int x_dt, const void* gm, const void* bt, void* y_row, int y_dt, void* y_fm) -> fsvd_status {
    LayerNormArgs la{};
    la.X = x; la.x_dt = x_dt; la.gamma = gm; la.beta = bt; la.p_dt = io; la.eps = d->ln_eps;
    la.T = T; la.D = D; la.Yrow = y_row; la.yrow_dt = y_dt; la.Yfm = y_fm;
    FSVD_HIP(launch_layernorm(la, s));
    return FSVD_OK;
  };

  if (d->norm == FSVD_NORM_POST_LN) {
    // S1 = X + Attn(X) (fp32 stream) -> Y1 = LN1(S1) in place + FM copy -> S2 = Y1 + FFN(Y1) in place -> out = LN2(S2)
    FSVD_HIP(launch_pack_fm(X, io, T, D, c_buf, s));
    // (each LayerNorm is fused into the projection before it when that projection's V is prepacked and D allows)
    LnFuse f1{g1, b1, d->ln_eps, stream_buf, DT_F32, c_buf, false};
    FSVD_TRY(run_attention(d, c_buf, q, k, v, o, X, io, stream_buf, DT_F32, false, c_buf, rank_buf, s, per_head, &f1));
    if (!f1.done) FSVD_TRY(ln(stream_buf, DT_F32, g1, b1, stream_buf, DT_F32, c_buf));
    LnFuse f2{g2, b2, d->ln_eps, out, d->out_dtype, nullptr, false};
    FSVD_TRY(run_ffn(d, c_buf, LAYOUT_FM, DT_F16, w1, w2, stream_buf, DT_F32, stream_buf, DT_F32, rank_buf, s, &f2));
    if (!f2.done) FSVD_TRY(ln(stream_buf, DT_F32, g2, b2, out, d->out_dtype, nullptr));
  } else if (d->norm == FSVD_NORM_PRE_LN) {
    // N1 = LN1(X) (FM) -> X1 = X + Attn(N1) (fp32 stream) -> N2 = LN2(X1) (FM) -> out = X1 + FFN(N2)
    FSVD_TRY(ln(X, io, g1, b1, nullptr, 0, c_buf));
    FSVD_TRY(run_attention(d, c_buf, q, k, v, o, X, io, stream_buf, DT_F32, false, c_buf, rank_buf, s, per_head));
    FSVD_TRY(ln(stream_buf, DT_F32, g2, b2, nullptr, 0, c_buf));
    FSVD_TRY(run_ffn(d, c_buf, LAYOUT_FM, DT_F16, w1, w2, stream_buf, DT_F32, out, d->out_dtype, rank_buf, s));
  } else {
    // out = FFN(Attn(X)): the attention output goes straight into the FM buffer that feeds the FFN
    FSVD_HIP(launch_pack_fm(X, io, T, D, c_buf, s));
    FSVD_TRY(run_attention(d, c_buf, q, k, v, o, nullptr, 0, c_buf, DT_F16, true, c_buf, rank_buf, s, per_head));
    FSVD_TRY(run_ffn(d, c_buf, LAYOUT_FM, DT_F16, w1, w2, nullptr, 0, out, d->out_dtype, rank_buf, s));
  }
  return FSVD_OK;
}
}  // namespace

extern "C" {

fsvd_status fsvd_layer(const fsvd_desc* d, const void* X, const fsvd_factor* q, const fsvd_factor* k,
                       const fsvd_factor* v, const fsvd_factor* o, const void* g1, const void* b1,
                       const fsvd_factor* w1, const fsvd_factor* w2, const void* g2, const void* b2, void* out,
                       void* ws, size_t ws_bytes, void* stream) {
  return layer_impl(d, X, q, k, v, o, g1, b1, w1, w2, g2, b2, out, ws, ws_bytes, stream, false);
}

size_t fsvd_layer_groups_workspace(const fsvd_desc* d, int32_t groups, int32_t rq, int32_t rk, int32_t rv, int32_t ro, int32_t r1,
                                   int32_t r2) {
  if (check_desc(d, true) != FSVD_OK) return 0;
  if (check_rank(rq) || check_rank(rk) || check_rank(rv) || check_rank(ro) || check_rank(r1) || check_rank(r2)) return 0;
  const size_t G = groups > 0 ? groups : d->H;
  if (groups < 0 || d->H % G != 0) return 0;
  return plan_layer(d, G * rq, G * rk, G * rv, ro, r1, r2).total;
}
size_t fsvd_layer_heads_workspace(const fsvd_desc* d, int32_t rq, int32_t rk, int32_t rv, int32_t ro, int32_t r1, int32_t r2) {
  return fsvd_layer_groups_workspace(d, 0, rq, rk, rv, ro, r1, r2);
}

fsvd_status fsvd_layer_heads(const fsvd_desc* d, const void* X, const fsvd_factor* q, const fsvd_factor* k,
                             const fsvd_factor* v, const fsvd_factor* o, const void* g1, const void* b1,
                             const fsvd_factor* w1, const fsvd_factor* w2, const void* g2, const void* b2, void* out,
                             void* ws, size_t ws_bytes, void* stream) {
  return layer_impl(d, X, q, k, v, o, g1, b1, w1, w2, g2, b2, out, ws, ws_bytes, stream, true);
}

// ------------------------------------------------------------------ building blocks
namespace {
fsvd_status linear_impl(int32_t T, int32_t K, int32_t N, const void* A, fsvd_dtype a_dtype, const void* W,
                        const void* bias, fsvd_dtype w_dtype, const void* residual, fsvd_dtype r_dtype, void* C,
                        fsvd_dtype c_dtype, void* stream, bool tiled) {
  if (T <= 0 || K <= 0 || N <= 0 || !A || !W || !C) return FSVD_ERR_INVALID_ARG;
  if (mis16(A) || mis16(W) || mis16(C) || mis16(bias) || mis16(residual)) return FSVD_ERR_INVALID_ARG;
  if (!dtype_ok(a_dtype) || !dtype_ok16(w_dtype) || !dtype_ok(c_dtype) || (residual && !dtype_ok(r_dtype))) return FSVD_ERR_INVALID_ARG;
  if (K % 16 != 0 || N % 16 != 0) return FSVD_ERR_UNSUPPORTED;
  if ((long long)T * (K > N ? K : N) >= (1LL << 29)) return FSVD_ERR_UNSUPPORTED;
  LinearArgs a{};
  a.A = A; a.a_layout = LAYOUT_ROW; a.lda = K; a.a_dt = a_dtype; a.T = T; a.K = K; a.w_dt = w_dtype; a.w_tiled = tiled;
  a.c_layout = LAYOUT_ROW; a.c_dt = c_dtype; a.R = residual; a.ldr = N; a.r_dt = r_dtype; a.ngroups = 1;
  a.g[0] = {W, bias, C, N, N, N};
  FSVD_HIP(launch_linear(a, (hipStream_t)stream));
  return FSVD_OK;
}
}  // namespace

fsvd_status fsvd_linear(int32_t T, int32_t K, int32_t N, const void* A, fsvd_dtype a_dtype, const void* W,
                        const void* bias, fsvd_dtype w_dtype, const void* residual, fsvd_dtype r_dtype, void* C,
                        fsvd_dtype c_dtype, void* stream) {
  return linear_impl(T, K, N, A, a_dtype, W, bias, w_dtype, residual, r_dtype, C, c_dtype, stream, false);
}
fsvd_status fsvd_linear_tiled(int32_t T, int32_t K, int32_t N, const void* A, fsvd_dtype a_dtype, const void* W_tiled,
                              const void* bias, fsvd_dtype bias_dtype, const void* residual, fsvd_dtype r_dtype, void* C,
                              fsvd_dtype c_dtype, void* stream) {
  return linear_impl(T, K, N, A, a_dtype, W_tiled, bias, bias_dtype, residual, r_dtype, C, c_dtype, stream, true);
}

size_t fsvd_fm_bytes(int32_t T, int32_t K) {
  if (T <= 0 || K <= 0 || K % 8 != 0) return 0;
  return fm_bytes((size_t)T, (size_t)K);
}

fsvd_status fsvd_pack_fm(int32_t T, int32_t K, const void* src, fsvd_dtype src_dtype, void* dst_fm, void* stream) {
  if (T <= 0 || K <= 0 || !src || !dst_fm || !dtype_ok(src_dtype) || mis16(src) || mis16(dst_fm)) return FSVD_ERR_INVALID_ARG;
  if (K % 8 != 0 || fm_bytes(T, K) >= (1ULL << 31)) return FSVD_ERR_UNSUPPORTED;
  FSVD_HIP(launch_pack_fm(src, src_dtype, T, K, dst_fm, (hipStream_t)stream));
  return FSVD_OK;
}

size_t fsvd_tiled_bytes(int32_t rows, int32_t cols) {
  if (rows <= 0 || cols <= 0 || cols % 8 != 0) return 0;
  const size_t n = tiled_bytes(rows, cols);
  return n < ((size_t)1 << 31) ? n : 0;
}
fsvd_status fsvd_pack_tiled(int32_t rows, int32_t cols, const void* src, fsvd_dtype src_dtype, void* dst, void* stream) {
  if (rows <= 0 || cols <= 0 || !src || !dst || !dtype_ok16(src_dtype) || mis16(src) || mis16(dst)) return FSVD_ERR_INVALID_ARG;
  if (!fsvd_tiled_bytes(rows, cols)) return FSVD_ERR_UNSUPPORTED;
  FSVD_HIP(launch_pack_tiled(src, src_dtype, rows, cols, dst, (hipStream_t)stream));
  return FSVD_OK;
}

fsvd_status fsvd_unpack_fm(int32_t T, int32_t K, const void* src_fm, void* dst, fsvd_dtype dst_dtype, void* stream) {
  if (T <= 0 || K <= 0 || !src_fm || !dst || !dtype_ok(dst_dtype) || mis16(src_fm) || mis16(dst)) return FSVD_ERR_INVALID_ARG;
  if (K % 8 != 0 || fm_bytes(T, K) >= (1ULL << 31)) return FSVD_ERR_UNSUPPORTED;
  FSVD_HIP(launch_unpack_fm(src_fm, T, K, dst, dst_dtype, (hipStream_t)stream));
  return FSVD_OK;
}

namespace {
fsvd_status attention_core_impl(const fsvd_desc* d, const void* Pq, const void* Pk, const void* Pv, const fsvd_factor* q,
                                const fsvd_factor* k, const fsvd_factor* v, void* context, void* stream, bool per_head) {
  FSVD_TRY(check_desc(d, false));
  const int tiled_ok = per_head ? 1 : 3;   // the U members are not read here: any layout value is accepted for them
  FSVD_TRY(check_factor(q, d->D, d->D, false, true, tiled_ok));
  FSVD_TRY(check_factor(k, d->D, d->D, false, true, tiled_ok));
  FSVD_TRY(check_factor(v, d->D, d->D, false, true, tiled_ok));
  if (q->v_layout != k->v_layout || q->v_layout != v->v_layout) return FSVD_ERR_UNSUPPORTED;
  if (!Pq || !Pk || !Pv || !context || mis16(Pq) || mis16(Pk) || mis16(Pv) || mis16(context)) return FSVD_ERR_INVALID_ARG;
  AttnCoreArgs ca{};
  ca.Pq = Pq; ca.Pk = Pk; ca.Pv = Pv;
  if (per_head && (q->groups < 0 || d->H % groups_of(d, q) != 0 || k->groups != q->groups || v->groups != q->groups))
    return FSVD_ERR_INVALID_ARG;
  ca.rq = q->rank; ca.rk = k->rank; ca.rv = v->rank; ca.per_head = per_head ? d->H / groups_of(d, q) : 0;
  ca.Vq = q->V; ca.Vk = k->V; ca.Vv = v->V; ca.bq = q->bias; ca.bk = k->bias; ca.bv = v->bias;
  ca.w_dt = d->io_dtype; ca.tiled = q->v_layout == FSVD_TILED; ca.B = d->B; ca.M = d->M; ca.D = d->D; ca.H = d->H;
  ca.causal = d->causal; ca.key_len = d->key_len; ca.scale = resolve_scale(d);
  ca.C = context;
  FSVD_HIP(launch_attn_core(ca, (hipStream_t)stream));
  return FSVD_OK;
}
}  // namespace

fsvd_status fsvd_attention_core(const fsvd_desc* d, const void* Pq, const void* Pk, const void* Pv, const fsvd_factor* q,
                                const fsvd_factor* k, const fsvd_factor* v, void* context, void* stream) {
  return attention_core_impl(d, Pq, Pk, Pv, q, k, v, context, stream, false);
}
fsvd_status fsvd_attention_heads_core(const fsvd_desc* d, const void* Pq, const void* Pk, const void* Pv,
                                      const fsvd_factor* q, const fsvd_factor* k, const fsvd_factor* v, void* context,
                                      void* stream) {
  return attention_core_impl(d, Pq, Pk, Pv, q, k, v, context, stream, true);
}

size_t fsvd_ffn_core_workspace(const fsvd_desc* d, int32_t r1, int32_t r2) {
  if (check_desc(d, true) != FSVD_OK) return 0;
  if (check_rank(r1) || check_rank(r2)) return 0;
  return align_up(ffn_core_partial_bytes(d->B * d->M, r1, r2, d->F));
}

fsvd_status fsvd_ffn_core(const fsvd_desc* d, const void* P1, const fsvd_factor* w1, const fsvd_factor* w2, void* Z,
                          void* ws, size_t ws_bytes, void* stream) {
  FSVD_TRY(check_desc(d, true));
  FSVD_TRY(check_factor(w1, d->D, d->F, false, true, 3));   // U of w1 and V of w2 are not read here
  FSVD_TRY(check_factor(w2, d->F, d->D, true, false, 3));
  if (w1->v_layout != w2->u_layout) return FSVD_ERR_UNSUPPORTED;
  if (!P1 || !Z || mis16(P1) || mis16(Z)) return FSVD_ERR_INVALID_ARG;
  const size_t need = fsvd_ffn_core_workspace(d, w1->rank, w2->rank);
  if (need) FSVD_TRY(check_ws(ws, ws_bytes, need));
  FfnCoreArgs fa{};
  fa.P1 = P1; fa.r1 = w1->rank; fa.V1 = w1->V; fa.b1 = w1->bias; fa.U2 = w2->U;
  fa.r2 = w2->rank; fa.w_dt = d->io_dtype; fa.tiled = w1->v_layout == FSVD_TILED; fa.T = d->B * d->M; fa.F = d->F;
  fa.act = d->act; fa.Z = Z; fa.Zpart = need ? (float*)ws : nullptr;
  FSVD_HIP(launch_ffn_core(fa, (hipStream_t)stream));
  return FSVD_OK;
}

// ------------------------------------------------------------------------------------------------------------
// Decoding step against a rank-space KV cache
// ------------------------------------------------------------------------------------------------------------
namespace {
int decode_nsplit(int B) {          // parts the keys of one sequence are split into: about one workgroup per compute unit
  int n = 256 / (B > 0 ? B : 1);
  return n < 1 ? 1 : (n > 32 ? 32 : n);
}
fsvd_status check_decode_shape(const fsvd_desc* d, int r_k, int r_v) {
  if (!d || d->M <= 0) return FSVD_ERR_INVALID_ARG;
  fsvd_desc one = *d;      // M is the cache capacity here, not a dimension of a [B, M, D] tensor: the tensors are [B, D]
  one.M = 1;
  FSVD_TRY(check_desc(&one, false));
  if (r_k <= 0 || r_v <= 0) return FSVD_ERR_INVALID_ARG;
  if (r_k % 64 != 0 || r_v % 32 != 0 || r_k > 1024 || r_v > 1024 || d->H > 32) return FSVD_ERR_UNSUPPORTED;
  if (fm_bytes(d->M, r_k) >= ((size_t)1 << 31) || decode_vcache_seq_bytes(d->M, r_v) >= ((size_t)1 << 31)) return FSVD_ERR_UNSUPPORTED;
  return FSVD_OK;
}
struct DecodeCorePlan { size_t stats, upart, total; int nsplit; };
DecodeCorePlan plan_decode_core(int B, int r_v) {
  DecodeCorePlan pl;
  pl.nsplit = decode_nsplit(B);
  pl.stats = 0;
  pl.upart = align_up((size_t)B * pl.nsplit * 64 * 4);
  pl.total = pl.upart + align_up((size_t)B * pl.nsplit * r_v * 32 * 2);
  return pl;
}
constexpr int kDecodeKParts = 16;     // room for this many partial results of a projection whose contraction is split
struct DecodePlan { size_t pq, pk, pv, qf, w, nk, u, ctx, to, core, part, part_bytes, total; };
DecodePlan plan_decode(const fsvd_desc* d, int rq, int rk, int rv, int ro) {
  const size_t B = d->B, D = d->D;
  DecodePlan pl;
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t at = off; off += align_up(bytes); return at; };
  pl.pq = take(B * rq * 2); pl.pk = take(B * rk * 2); pl.pv = take(B * rv * 2);
  pl.qf = take(B * D * 2);
  pl.w = take(B * (size_t)((rk + 63) / 64) * 4096);
  pl.nk = take(B * 4);
  pl.u = take(B * d->H * (size_t)rv * 4);
  pl.ctx = take(B * D * 2);
  pl.to = take(B * ro * 2);
  pl.core = take(plan_decode_core(d->B, rv).total);
  const size_t widest = smax(smax((size_t)rq + rk + rv, D), (size_t)ro);
  pl.part_bytes = (size_t)kDecodeKParts * B * widest * 4;
  pl.part = take(pl.part_bytes);
  pl.total = off;
  return pl;
}
fsvd_status run_decode_core(const fsvd_desc* d, int r_k, int r_v, const void* W, const void* kc, const void* vc,
                            const int32_t* n_keys, float* u_out, char* ws, hipStream_t s) {
  const DecodeCorePlan pl = plan_decode_core(d->B, r_v);
  DecodeCoreArgs ca{};
  ca.W = W; ca.kcache = kc; ca.vcache = vc; ca.n_keys = n_keys;
  ca.B = d->B; ca.t_max = d->M; ca.r_k = r_k; ca.r_v = r_v; ca.nsplit = pl.nsplit;
  ca.stats = (float*)(ws + pl.stats); ca.upart = (_Float16*)(ws + pl.upart);
  FSVD_HIP(launch_decode_core(ca, s));
  FSVD_HIP(launch_decode_merge(ca.stats, ca.upart, n_keys, d->B, d->M, pl.nsplit, d->H, r_v, u_out, s));
  return FSVD_OK;
}
}  // namespace

size_t fsvd_decode_kcache_bytes(int32_t B, int32_t t_max, int32_t r_k) {
  if (B <= 0 || t_max <= 0 || r_k <= 0 || r_k % 64 != 0) return 0;
  return (size_t)B * fm_bytes(t_max, r_k);
}
size_t fsvd_decode_vcache_bytes(int32_t B, int32_t t_max, int32_t r_v) {
  if (B <= 0 || t_max <= 0 || r_v <= 0 || r_v % 32 != 0) return 0;
  return (size_t)B * decode_vcache_seq_bytes(t_max, r_v);
}
fsvd_status fsvd_decode_cache_write(int32_t B, int32_t t_max, int32_t r, int32_t n_new, const int32_t* t_start, const void* P_new,
                                    int32_t which, void* cache, void* stream) {
  if (B <= 0 || t_max <= 0 || r <= 0 || n_new <= 0 || !t_start || !P_new || !cache || (which != 0 && which != 1)) return FSVD_ERR_INVALID_ARG;
  if (mis16(P_new) || mis16(cache)) return FSVD_ERR_INVALID_ARG;
  if (r % (which == 0 ? 64 : 32) != 0) return FSVD_ERR_UNSUPPORTED;
  if ((size_t)B * n_new * r >= ((size_t)1 << 31)) return FSVD_ERR_UNSUPPORTED;
  FSVD_HIP(launch_decode_cache_write(P_new, t_start, B, t_max, r, n_new, which, cache, (hipStream_t)stream));
  return FSVD_OK;
}

size_t fsvd_decode_core_workspace(const fsvd_desc* d, int32_t r_k, int32_t r_v) {
  if (check_decode_shape(d, r_k, r_v) != FSVD_OK) return 0;
  return plan_decode_core(d->B, r_v).total;
}
fsvd_status fsvd_decode_attention_core(const fsvd_desc* d, int32_t r_k, int32_t r_v, const void* W, const void* kcache,
                                       const void* vcache, const int32_t* n_keys, void* u_out, void* ws, size_t ws_bytes,
                                       void* stream) {
  FSVD_TRY(check_decode_shape(d, r_k, r_v));
  if (!W || !kcache || !vcache || !n_keys || !u_out) return FSVD_ERR_INVALID_ARG;
  if (mis16(W) || mis16(kcache) || mis16(vcache) || mis16(u_out)) return FSVD_ERR_INVALID_ARG;
  FSVD_TRY(check_ws(ws, ws_bytes, plan_decode_core(d->B, r_v).total));
  return run_decode_core(d, r_k, r_v, W, kcache, vcache, n_keys, (float*)u_out, (char*)ws, (hipStream_t)stream);
}

size_t fsvd_decode_attention_workspace(const fsvd_desc* d, int32_t rq, int32_t rk, int32_t rv, int32_t ro) {
  if (check_decode_shape(d, rk, rv) != FSVD_OK) return 0;
  if (check_rank(rq) || check_rank(ro)) return 0;
  return plan_decode(d, rq, rk, rv, ro).total;
}
fsvd_status fsvd_decode_attention(const fsvd_desc* d, const void* x_new, const fsvd_factor* q, const fsvd_factor* k,
                                  const fsvd_factor* v, const fsvd_factor* o, void* kcache, void* vcache,
                                  const int32_t* t_len, void* out, void* ws, size_t ws_bytes, void* stream) {
  if (!d) return FSVD_ERR_INVALID_ARG;
  FSVD_TRY(check_factor(q, d->D, d->D, true, true, 3));
  FSVD_TRY(check_factor(k, d->D, d->D, true, true, 1));     // V of k and v is read row by row by the kernels of this step
  FSVD_TRY(check_factor(v, d->D, d->D, true, true, 1));
  FSVD_TRY(check_factor(o, d->D, d->D, true, true, 3));
  if (q->u_layout != k->u_layout || q->u_layout != v->u_layout) return FSVD_ERR_UNSUPPORTED;   // one projection launch
  FSVD_TRY(check_decode_shape(d, k->rank, v->rank));
  if (!x_new || !kcache || !vcache || !t_len || !out) return FSVD_ERR_INVALID_ARG;
  if (mis16(x_new) || mis16(kcache) || mis16(vcache) || mis16(out)) return FSVD_ERR_INVALID_ARG;
  const DecodePlan pl = plan_decode(d, q->rank, k->rank, v->rank, o->rank);
  FSVD_TRY(check_ws(ws, ws_bytes, pl.total));
  char* w = (char*)ws;
  hipStream_t s = (hipStream_t)stream;
  const int B = d->B, D = d->D;

  LinearArgs p{};       // rank projections of the new tokens, row-major fp16
  p.A = x_new; p.a_layout = LAYOUT_ROW; p.lda = D; p.a_dt = d->io_dtype; p.T = B; p.K = D; p.w_dt = d->io_dtype;
  p.w_tiled = q->u_layout == FSVD_TILED; p.c_layout = LAYOUT_ROW; p.c_dt = DT_F16; p.ngroups = 3;
  p.g[0] = {q->U, nullptr, w + pl.pq, q->rank, q->rank, q->rank};
  p.g[1] = {k->U, nullptr, w + pl.pk, k->rank, k->rank, k->rank};
  p.g[2] = {v->U, nullptr, w + pl.pv, v->rank, v->rank, v->rank};
  p.part = (float*)(w + pl.part); p.part_bytes = pl.part_bytes; p.ldp = q->rank + k->rank + v->rank;
  FSVD_HIP(launch_linear(p, s));
  FSVD_HIP(launch_decode_append(w + pl.pk, w + pl.pv, t_len, B, d->M, k->rank, v->rank, kcache, vcache, (int32_t*)(w + pl.nk), s));

  LinearArgs qa{};      // the new queries at full width, fp16
  qa.A = w + pl.pq; qa.a_layout = LAYOUT_ROW; qa.lda = q->rank; qa.a_dt = DT_F16; qa.T = B; qa.K = q->rank; qa.w_dt = d->io_dtype;
  qa.w_tiled = q->v_layout == FSVD_TILED; qa.c_layout = LAYOUT_ROW; qa.c_dt = DT_F16; qa.ngroups = 1;
  qa.g[0] = {q->V, q->bias, w + pl.qf, D, D, D};
  qa.part = (float*)(w + pl.part); qa.part_bytes = pl.part_bytes; qa.ldp = D;
  FSVD_HIP(launch_linear(qa, s));
  FSVD_HIP(launch_decode_absorb(w + pl.qf, k->V, d->io_dtype, B, D, d->H, k->rank, resolve_scale(d), w + pl.w, s));
  FSVD_TRY(run_decode_core(d, k->rank, v->rank, w + pl.w, kcache, vcache, (const int32_t*)(w + pl.nk), (float*)(w + pl.u),
                           w + pl.core, s));
  FSVD_HIP(launch_decode_value((const float*)(w + pl.u), v->V, v->bias, d->io_dtype, B, D, d->H, v->rank, w + pl.ctx, s));

  LinearArgs oa{};      // factored output projection
  oa.A = w + pl.ctx; oa.a_layout = LAYOUT_ROW; oa.lda = D; oa.a_dt = DT_F16; oa.T = B; oa.K = D; oa.w_dt = d->io_dtype;
  oa.w_tiled = o->u_layout == FSVD_TILED; oa.c_layout = LAYOUT_ROW; oa.c_dt = DT_F16; oa.ngroups = 1;
  oa.g[0] = {o->U, nullptr, w + pl.to, o->rank, o->rank, o->rank};
  oa.part = (float*)(w + pl.part); oa.part_bytes = pl.part_bytes; oa.ldp = o->rank;
  FSVD_HIP(launch_linear(oa, s));
  LinearArgs ob{};
  ob.A = w + pl.to; ob.a_layout = LAYOUT_ROW; ob.lda = o->rank; ob.a_dt = DT_F16; ob.T = B; ob.K = o->rank; ob.w_dt = d->io_dtype;
  ob.w_tiled = o->v_layout == FSVD_TILED; ob.c_layout = LAYOUT_ROW; ob.c_dt = d->out_dtype; ob.ngroups = 1;
  ob.g[0] = {o->V, o->bias, out, D, D, D};
  ob.part = (float*)(w + pl.part); ob.part_bytes = pl.part_bytes; ob.ldp = D;
  FSVD_HIP(launch_linear(ob, s));
  return FSVD_OK;
}

fsvd_status fsvd_mfma_probe(int32_t workgroups, int32_t iters, void* out, void* stream) {
  if (!out || mis16(out)) return FSVD_ERR_INVALID_ARG;
  if (workgroups < 1 || workgroups > 65536 || iters < 1 || iters > (1 << 20)) return FSVD_ERR_INVALID_ARG;
  FSVD_HIP(launch_mfma_probe(workgroups, iters, (float*)out, (hipStream_t)stream));
  return FSVD_OK;
}

fsvd_status fsvd_dma_probe(int32_t workgroups, int32_t steps, int32_t with_work, const void* src, size_t region_bytes, void* out,
                           void* stream) {
  if (!src || !out || mis16(src) || mis16(out)) return FSVD_ERR_INVALID_ARG;
  if (workgroups < 1 || workgroups > 65536 || steps < 1 || steps > (1 << 20)) return FSVD_ERR_INVALID_ARG;
  if (region_bytes == 0 || region_bytes % 32768 != 0 || region_bytes > ((size_t)1 << 30)) return FSVD_ERR_INVALID_ARG;
  FSVD_HIP(launch_dma_probe(workgroups, steps, with_work, src, (unsigned)region_bytes, (float*)out, (hipStream_t)stream));
  return FSVD_OK;
}

fsvd_status fsvd_layernorm(int32_t T, int32_t D, const void* X, fsvd_dtype x_dtype, const void* gamma, const void* beta,
                           fsvd_dtype p_dtype, float eps, void* Y, fsvd_dtype y_dtype, void* stream) {
  if (T <= 0 || D <= 0 || !X || !gamma || !beta || !Y) return FSVD_ERR_INVALID_ARG;
  if (mis16(X) || mis16(gamma) || mis16(beta) || mis16(Y)) return FSVD_ERR_INVALID_ARG;
  if (!dtype_ok(x_dtype) || !dtype_ok(p_dtype) || !dtype_ok(y_dtype) || !(eps >= 0.f)) return FSVD_ERR_INVALID_ARG;
  if (D > 8192 || D % 8 != 0) return FSVD_ERR_UNSUPPORTED;
  if ((long long)T * D >= (1LL << 31)) return FSVD_ERR_UNSUPPORTED;
  LayerNormArgs la{};
  la.X = X; la.x_dt = x_dtype; la.gamma = gamma; la.beta = beta; la.p_dt = p_dtype; la.eps = eps;
  la.T = T; la.D = D; la.Yrow = Y; la.yrow_dt = y_dtype; la.Yfm = nullptr;
  FSVD_HIP(launch_layernorm(la, (hipStream_t)stream));
  return FSVD_OK;
}

}  // extern "C"
