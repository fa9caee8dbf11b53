"""Plain CPU oracle of one SVD-compressed transformer layer.  TEST INFRASTRUCTURE ONLY.

This is the unfused definition of what the streaming kernels compute.  The
paper's method is a re-scheduling of this computation (tile-by-tile rebuild of
Q/K/V and of the FFN hidden activation), not an approximation of it, so the
oracle is the definition written out: every intermediate is materialised at
full width, in float64, with numpy's matmul as the only library step.  No
tiling, no fusion, no online softmax.

It shares no code with the GPU library and imports nothing from it.  It is
used by tests/, by the smoke check and by the benchmark's cpu_baseline leg,
and by nothing on the product path.

Parity pins (tests/test_oracle_pins.py): full-rank identity against a dense
layer written with torch's library routines, the Eckart-Young closed form for
truncation, brute-force attention with python loops on tiny shapes, softmax /
GELU / LayerNorm closed forms, mask and bias invariants; the decoding step
against the last row of causal attention over the whole sequence.  The whole layer at
benchmark sizes has no printed values in the paper to compare against: beyond
those pins it is "parity unpinned".

Notation follows the paper: X [B, M, D]; per projection a in {q, k, v, o} the
factors U_a [D, r], V_a [r, D] and bias b_a [D]; P_a = X U_a; H heads of width
d_h = D / H; FFN factors (U_i, V_i, b_i) and (U_o, V_o, b_o).
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf as _erf

F64 = np.float64


def _f64(a):
    return None if a is None else np.asarray(a, dtype=F64)


# ---------------------------------------------------------------------------
# factored projection  (Methodology: W^[r] = U~ V~^T; FlashSVDAttention text:
# P_a = X U_a, tile = P_a V_a + b_a)
# ---------------------------------------------------------------------------

def rank_projection(x, U):
    """P = X U: the rank-space activation, [..., r]."""
    return _f64(x) @ _f64(U)


def factored_linear(x, fac):
    """(X U) V + b for a factor dict {"U", "V", "b"}; b may be None."""
    y = rank_projection(x, fac["U"]) @ _f64(fac["V"])
    if fac.get("b") is not None:
        y = y + _f64(fac["b"])
    return y


# ---------------------------------------------------------------------------
# element-wise pieces
# ---------------------------------------------------------------------------

def gelu_erf(x):
    """Exact GELU, 0.5 x (1 + erf(x / sqrt 2))."""
    x = _f64(x)
    return 0.5 * x * (1.0 + _erf(x / np.sqrt(2.0)))


def gelu_tanh(x):
    """Tanh form of GELU, 0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3))) (the "arbitrary phi" of FlashSVDFFN V1)."""
    x = _f64(x)
    return 0.5 * x * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (x + 0.044715 * x ** 3)))


def activation(x, act="gelu_erf"):
    if act == "gelu_erf":
        return gelu_erf(x)
    if act == "gelu_tanh":
        return gelu_tanh(x)
    if act == "relu":
        return np.maximum(_f64(x), 0.0)
    raise ValueError(act)


def layer_norm(x, gamma, beta, eps):
    """Per-token LayerNorm with the biased variance."""
    x = _f64(x)
    mean = x.mean(axis=-1, keepdims=True)
    var = ((x - mean) ** 2).mean(axis=-1, keepdims=True)
    return (x - mean) / np.sqrt(var + eps) * _f64(gamma) + _f64(beta)


def softmax_rows(scores):
    """Row-wise softmax of a score matrix whose masked entries are -inf."""
    m = scores.max(axis=-1, keepdims=True)
    p = np.exp(scores - m)
    return p / p.sum(axis=-1, keepdims=True)


# ---------------------------------------------------------------------------
# attention  (Alg. 1 Part II computes exactly this, block by block; Definition
# "Attention Activation Approximation" for the head split)
# ---------------------------------------------------------------------------

def attention_context_one_sequence(x, q, k, v, H, causal=False, key_len=None, scale=None,
                                   rows=None):
    """Context C [M or len(rows), D] of one sequence x [M, D].

    Q = (x U_q) V_q + b_q, same for K and V; columns [h d_h, (h+1) d_h) belong to
    head h; per head S = Q_h K_h^T * scale (scale = 1/sqrt(d_h) by default);
    key j is masked (score -inf) when j >= key_len or, if causal, j > i;
    alpha = softmax over keys; C_h = alpha V_h; heads are concatenated.
    ``rows`` restricts the *query* rows that are evaluated (keys always span the
    whole sequence); it exists so that sampled rows of a long sequence can be
    checked without forming every M x M score matrix.
    """
    x = _f64(x)
    M = x.shape[0]
    D = np.shape(q["V"])[1]          # width of the rebuilt Q/K/V (x itself may be any width)
    d_h = D // H
    if scale is None or scale == 0:
        scale = 1.0 / np.sqrt(d_h)
    rows = np.arange(M) if rows is None else np.asarray(rows, dtype=np.int64)
    Q = factored_linear(x[rows], q)
    K = factored_linear(x, k)
    V = factored_linear(x, v)
    key_idx = np.arange(M)
    masked = np.zeros((len(rows), M), dtype=bool)
    if key_len is not None:
        masked |= (key_idx >= int(key_len))[None, :]
    if causal:
        masked |= key_idx[None, :] > rows[:, None]
    C = np.empty((len(rows), D), dtype=F64)
    for h in range(H):
        sl = slice(h * d_h, (h + 1) * d_h)
        S = (Q[:, sl] @ K[:, sl].T) * scale
        S[masked] = -np.inf
        C[:, sl] = softmax_rows(S) @ V[:, sl]
    return C


def attention(X, q, k, v, o, H, causal=False, key_len=None, scale=None):
    """Attention block output A = (C U_o) V_o + b_o for X [B, M, D]."""
    X = _f64(X)
    B = X.shape[0]
    out = np.empty_like(X)
    for b in range(B):
        kl = None if key_len is None else key_len[b]
        C = attention_context_one_sequence(X[b], q, k, v, H, causal, kl, scale)
        out[b] = factored_linear(C, o)
    return out


# ---------------------------------------------------------------------------
# decoding with a rank-space KV cache  (appendix on decoder models, paragraphs
# "Prefill" / "Decoding Phase": the cache holds the rank-space keys and values
# P_k, P_v [B, t, r] instead of K, V [B, t, D]; step t attends one new query
# against the cached rows and its own)
# ---------------------------------------------------------------------------

def decode_attention(x_new, Pk_cache, Pv_cache, lens, q, k, v, o, H, scale=None):
    """One decoding step of the attention block.  x_new [B, D] is the new token of every sequence; Pk_cache [B, t_max, r_k]
    and Pv_cache [B, t_max, r_v] hold the rank-space keys / values of the lens[b] earlier tokens of sequence b (rows
    beyond lens[b] are ignored).  Returns (out [B, D], pk_new [B, r_k], pv_new [B, r_v]): the block's output for the
    new token and the two rows that extend the cache.

    Written as the plain definition, with nothing absorbed or reordered: the cached rows and the new row are turned back
    into full-width keys and values K = P_k V_k + b_k, V = P_v V_v + b_v, the new query is Q = (x U_q) V_q + b_q, and per
    head the new token attends to all lens[b] + 1 keys (itself included: the causal mask of the last row)."""
    x_new = _f64(x_new)
    B, D = x_new.shape[0], np.shape(q["V"])[1]
    d_h = D // H
    if scale is None or scale == 0:
        scale = 1.0 / np.sqrt(d_h)
    pq = rank_projection(x_new, q["U"])
    pk_new = rank_projection(x_new, k["U"])
    pv_new = rank_projection(x_new, v["U"])
    out = np.empty((B, D), dtype=F64)
    for b in range(B):
        n = int(lens[b])
        Pk = np.concatenate([_f64(Pk_cache[b, :n]), pk_new[b:b + 1]], axis=0)
        Pv = np.concatenate([_f64(Pv_cache[b, :n]), pv_new[b:b + 1]], axis=0)
        Qb = pq[b:b + 1] @ _f64(q["V"]) + (0.0 if q.get("b") is None else _f64(q["b"]))
        Kb = Pk @ _f64(k["V"]) + (0.0 if k.get("b") is None else _f64(k["b"]))
        Vb = Pv @ _f64(v["V"]) + (0.0 if v.get("b") is None else _f64(v["b"]))
        C = np.empty((1, D), dtype=F64)
        for h in range(H):
            sl = slice(h * d_h, (h + 1) * d_h)
            C[:, sl] = softmax_rows((Qb[:, sl] @ Kb[:, sl].T) * scale) @ Vb[:, sl]
        out[b] = factored_linear(C, o)[0]
    return out, pk_new, pv_new


# ---------------------------------------------------------------------------
# feed-forward  (Alg. 2 computes exactly this: P = X U_i, Y = phi(P V_i + b_i),
# Z = Y U_o in rank space, O = Z V_o + b_o)
# ---------------------------------------------------------------------------

def attention_per_head(X, q, k, v, o, H, causal=False, key_len=None, scale=None):
    """Attention block with per-head factors (the paper's own setting for attention: each head h has its rank-r pair
    U_a^(h) [D, r], V_a^(h) [r, d_h]; Sec. FlashSVDAttention / Alg. 1 with V_a in r x d_h): q, k, v hold
    U [D, H r] (head h = columns h r ..), V [H, r, d_h] and b [D]; o is a whole-matrix factor.

    Grouped heads (appendix, grouped-head compression: the H heads are compressed jointly in G groups of H / G heads,
    interpolating between one factor pair for all heads, G = 1, and one per head, G = H) are the same with
    V [G, r, D / G] and U [D, G r]: group g's pair rebuilds the D / G columns of its heads.  G is V.shape[0].

    Written as the plain definition: per group the full-width columns (X U_g) V_g + b_g, split into its heads; scores,
    masking and softmax per query row and head; heads concatenated; factored output projection."""
    X = _f64(X)
    B, M, D = X.shape
    d_h = D // H
    sc = (1.0 / np.sqrt(d_h)) if (scale is None or scale == 0) else float(scale)   # 0 selects the default, as in attention()
    out = np.empty((B, M, D), dtype=F64)

    def project(x, fac, h):
        G, r, width = np.shape(fac["V"])
        hpg = H // G                              # heads per group
        g, j = h // hpg, h % hpg
        y = ((x @ _f64(fac["U"])[:, g * r:(g + 1) * r]) @ _f64(fac["V"])[g])[:, j * d_h:(j + 1) * d_h]
        if fac.get("b") is not None:
            y = y + _f64(fac["b"])[h * d_h:(h + 1) * d_h]
        return y

    for b in range(B):
        ctx = np.empty((M, D), dtype=F64)
        n_keys = M if key_len is None else int(key_len[b])
        for h in range(H):
            Qh, Kh, Vh = project(X[b], q, h), project(X[b], k, h), project(X[b], v, h)
            S = (Qh @ Kh.T) * sc
            allowed = np.zeros((M, M), dtype=bool)
            allowed[:, :n_keys] = True
            if causal:
                allowed &= np.tril(np.ones((M, M), dtype=bool))
            S = np.where(allowed, S, -np.inf)
            ctx[:, h * d_h:(h + 1) * d_h] = softmax_rows(S) @ Vh
        out[b] = factored_linear(ctx, o)
    return out


def ffn(X, w1, w2, act="gelu_erf"):
    hidden = activation(factored_linear(X, w1), act)
    return factored_linear(hidden, w2)


# ---------------------------------------------------------------------------
# one layer  (residual / LayerNorm wiring is not part of the paper's method;
# post-LN is BERT's, pre-LN the decoder convention)
# ---------------------------------------------------------------------------

def layer(X, q, k, v, o, ln1, w1, w2, ln2, H, norm="post_ln", causal=False, key_len=None,
          scale=None, act="gelu_erf", eps=1e-5, per_head=False):
    """ln1/ln2 are (gamma, beta) pairs (ignored when norm == "none"); per_head: q, k, v hold per-head factors."""
    X = _f64(X)
    attn = attention_per_head if per_head else attention
    if norm == "post_ln":
        y1 = layer_norm(X + attn(X, q, k, v, o, H, causal, key_len, scale), *ln1, eps)
        return layer_norm(y1 + ffn(y1, w1, w2, act), *ln2, eps)
    if norm == "pre_ln":
        x1 = X + attn(layer_norm(X, *ln1, eps), q, k, v, o, H, causal, key_len, scale)
        return x1 + ffn(layer_norm(x1, *ln2, eps), w1, w2, act)
    if norm == "none":
        return ffn(attn(X, q, k, v, o, H, causal, key_len, scale), w1, w2, act)
    raise ValueError(norm)


def layer_rows(X, b, rows, q, k, v, o, ln1, w1, w2, ln2, H, norm="post_ln", causal=False,
               key_len=None, scale=None, act="gelu_erf", eps=1e-5, part="layer"):
    """Rows ``rows`` of sequence ``b`` of the layer (or of one block) output.

    Everything after the attention context is token-wise, so the sampled rows of
    a long sequence follow from that sequence's keys and values alone.
    part = "layer" | "attention" | "ffn".
    """
    x = _f64(X[b])
    rows = np.asarray(rows, dtype=np.int64)
    kl = None if key_len is None else key_len[b]

    def attn_rows(inp):
        C = attention_context_one_sequence(inp, q, k, v, H, causal, kl, scale, rows=rows)
        return factored_linear(C, o)

    if part == "attention":
        return attn_rows(x)
    if part == "ffn":
        return ffn(x[rows], w1, w2, act)
    if norm == "post_ln":
        y1 = layer_norm(x[rows] + attn_rows(x), *ln1, eps)
        return layer_norm(y1 + ffn(y1, w1, w2, act), *ln2, eps)
    if norm == "pre_ln":
        x1 = x[rows] + attn_rows(layer_norm(x, *ln1, eps))
        return x1 + ffn(layer_norm(x1, *ln2, eps), w1, w2, act)
    if norm == "none":
        return ffn(attn_rows(x), w1, w2, act)
    raise ValueError(norm)


# ---------------------------------------------------------------------------
# transient off-chip memory, in stored scalars  (Memory Complexity section:
# vanilla-SVD proposition, FlashSVDAttention theorem, FFN V1 theorem)
# ---------------------------------------------------------------------------

def attention_transient_scalars(B, M, D, H, r, streaming, with_scores=False):
    """Input-dependent attention intermediates, no buffer reuse.

    Streaming keeps only P_q, P_k, P_v (3 B M r).  The unfused factored layer
    also holds the rebuilt Q, K, V (3 B M D) and, without flash-style tiling,
    the B H M^2 score matrix.
    """
    n = 3 * B * M * r
    if not streaming:
        n += 3 * B * M * D
        if with_scores:
            n += B * H * M * M
    return n


def ffn_transient_scalars(B, M, F, r, streaming):
    """P and Z in rank space (2 B M r); the unfused path adds the B M F hidden."""
    n = 2 * B * M * r
    if not streaming:
        n += B * M * F
    return n


def attention_param_count(D, H, r=None, per_head=True, dense_out=True):
    """Stored parameters of one attention block, biases included.

    r is None: four dense D x D projections.  Otherwise q, k, v are factored,
    either per head (U [D, r] and V [r, d_h] for each of H heads; proof of MHA
    reduction efficiency) or as whole matrices (U [D, r], V [r, D]); the output
    projection stays dense or is factored as a whole matrix.
    """
    d_h = D // H
    if r is None:
        return 4 * D * D + 4 * D
    qkv = 3 * (H * (D * r + r * d_h) if per_head else (D * r + r * D)) + 3 * D
    out = (D * D if dense_out else 2 * D * r) + D
    return qkv + out
