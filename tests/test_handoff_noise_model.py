"""Where the error of the blocks comes from: a CPU model of the fp16 roundings on the HIP path.

Every contraction of the library runs on the fp16 matrix cores, so each tensor that is an MFMA operand is rounded to fp16
once: the rank-space activations (P_q, P_k, P_v, T_o = C U_o, P1, Z), the rebuilt Q/K/V tiles, the un-normalised
probabilities, the context C and the activated hidden chunk G.  This file evaluates the oracle's definition in float64
with exactly one (or all) of those roundings switched on and measures max|err| / RMS(ref) against the unrounded oracle,
on the first benchmark configuration (BERT-base width, 256 tokens).  It documents, reproducibly, why the stated 2e-3 is
applied to fsvd_layer (whose LayerNorms renormalise the output to unit RMS) and why the blocks called alone get their own
measured bounds: for the attention block the roundings no fp16-operand kernel can avoid (the rebuilt Q/K/V tiles and the
P operands of the rebuild) already exceed 2e-3 on their own.  Nothing here touches the GPU library.
"""
import numpy as np
import pytest

from oracle import fsvd_oracle as O
from paper_2508_01506_amd import workloads as W


def r16(x, on):
    return x.astype(np.float16).astype(np.float64) if on else x


def model_attention(inp, w, on):
    """The attention block of the oracle with fp16 rounding at the hand-offs named in `on`."""
    X = np.asarray(inp["X"], dtype=np.float64)
    B, M, D = X.shape
    H, dh = w.H, D // w.H
    out = np.empty_like(X)
    for b in range(B):
        proj = {}
        for a in "qkv":
            P = r16(O.rank_projection(X[b], inp[a]["U"]), "P" in on)
            proj[a] = P @ np.asarray(inp[a]["V"], dtype=np.float64) + np.asarray(inp[a]["b"], dtype=np.float64)
        scale = np.log2(np.e) / np.sqrt(dh)                      # the kernel folds the softmax scale into Q (log2 domain)
        Q, K, V = r16(proj["q"] * scale, "QKV" in on), r16(proj["k"], "QKV" in on), r16(proj["v"], "QKV" in on)
        C = np.empty((M, D))
        for h in range(H):
            sl = slice(h * dh, (h + 1) * dh)
            S = Q[:, sl] @ K[:, sl].T
            p = np.exp2(S - S.max(-1, keepdims=True))
            C[:, sl] = (r16(p, "prob" in on) @ V[:, sl]) / p.sum(-1, keepdims=True)
        To = r16(r16(C, "C" in on) @ np.asarray(inp["o"]["U"], dtype=np.float64), "To" in on)
        out[b] = To @ np.asarray(inp["o"]["V"], dtype=np.float64) + np.asarray(inp["o"]["b"], dtype=np.float64)
    return out


def model_ffn(inp, on):
    X = np.asarray(inp["X"], dtype=np.float64)
    P1 = r16(O.rank_projection(X, inp["w1"]["U"]), "P1" in on)
    G = r16(O.gelu_erf(P1 @ np.asarray(inp["w1"]["V"], dtype=np.float64) + inp["w1"]["b"]), "G" in on)
    Z = r16(G @ np.asarray(inp["w2"]["U"], dtype=np.float64), "Z" in on)
    return Z @ np.asarray(inp["w2"]["V"], dtype=np.float64) + inp["w2"]["b"]


def err(a, ref):
    return float(np.abs(a - ref).max() / np.sqrt(np.mean(ref ** 2)))


@pytest.fixture(scope="module")
def case():
    w = W.get_workload("cfg1_bert_base_b2_m128")
    inp = W.make_inputs(w)
    ref_a = O.attention(inp["X"], inp["q"], inp["k"], inp["v"], inp["o"], w.H)
    ref_f = O.ffn(inp["X"], inp["w1"], inp["w2"])
    return w, inp, ref_a, ref_f


def test_model_without_roundings_is_the_oracle(case):
    w, inp, ref_a, ref_f = case
    assert err(model_attention(inp, w, set()), ref_a) < 1e-12
    assert err(model_ffn(inp, set()), ref_f) < 1e-12


def test_attention_block_roundings_one_at_a_time(case):
    w, inp, ref_a, _ = case
    alone = {k: err(model_attention(inp, w, {k}), ref_a) for k in ("P", "QKV", "prob", "C", "To")}
    unavoidable = err(model_attention(inp, w, {"P", "QKV", "prob"}), ref_a)      # operands of the on-chip contractions
    everything = err(model_attention(inp, w, {"P", "QKV", "prob", "C", "To"}), ref_a)
    print("attention block, max|err|/RMS(ref) with one fp16 rounding switched on:",
          ", ".join(f"{k} {v:.2e}" for k, v in alone.items()),
          f"; P + QKV + prob {unavoidable:.2e}; all five {everything:.2e}")
    # every single rounding is a fraction of a per-mille; the score path (P and the Q/K/V tiles) is the largest
    assert all(2e-4 < v < 4e-3 for v in alone.values()), alone
    assert max(alone, key=alone.get) in ("P", "QKV")
    # the operands an fp16 matrix-core kernel cannot avoid rounding are, together, already beyond the 2e-3 of the layer gate
    assert unavoidable > 2e-3
    # all five agree with what the GPU measures on this workload (3.2e-3) to within the spread of a maximum
    assert 2e-3 < everything < 6e-3


def test_ffn_block_roundings_one_at_a_time(case):
    w, inp, _, ref_f = case
    alone = {k: err(model_ffn(inp, {k}), ref_f) for k in ("P1", "G", "Z")}
    everything = err(model_ffn(inp, {"P1", "G", "Z"}), ref_f)
    print("FFN block, max|err|/RMS(ref) with one fp16 rounding switched on:",
          ", ".join(f"{k} {v:.2e}" for k, v in alone.items()), f"; all three {everything:.2e}")
    assert all(4e-4 < v < 2e-3 for v in alone.values()), alone
    # three roundings of about 1e-3 each at the maximum: the block sits at the gate itself (the GPU measures 1.8e-3 here,
    # 1.8e-3 .. 2.2e-3 on the larger configurations and 3.3e-3 on the spectrum-built factors), hence its own test bound
    assert 1.2e-3 < everything < 2.5e-3
