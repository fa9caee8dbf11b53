"""Helpers shared by the GPU parity tests, the smoke check and the benchmark's checks.

The oracle side (numpy, float64) and the GPU side (libfsvd through the ctypes
binding) only meet here, on the same seeded inputs.
"""
from __future__ import annotations

import numpy as np

from oracle import fsvd_oracle as O
from paper_2508_01506_amd import workloads as W


def rel_err(got, ref) -> float:
    """max |got - ref| / RMS(ref): the parity metric."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.abs(got - ref).max() / np.sqrt(np.mean(ref ** 2)))


def oracle_call(inp, part="layer"):
    """Full oracle evaluation of one workload's inputs."""
    w = inp["workload"]
    a = (inp["q"], inp["k"], inp["v"], inp["o"])
    if part == "attention":
        fn = O.attention_per_head if w.r_head > 0 else O.attention
        return fn(inp["X"], *a, w.H, inp["causal"], inp["key_len"])
    if part == "ffn":
        return O.ffn(inp["X"], inp["w1"], inp["w2"])
    return O.layer(inp["X"], *a, (inp["ln1_gamma"], inp["ln1_beta"]), inp["w1"], inp["w2"],
                   (inp["ln2_gamma"], inp["ln2_beta"]), w.H, norm=w.norm, causal=inp["causal"],
                   key_len=inp["key_len"], eps=w.ln_eps, per_head=w.r_head > 0)


def oracle_rows(inp, b, rows, part="layer"):
    """Oracle evaluation of sampled rows of sequence b (for benchmark-size workloads)."""
    w = inp["workload"]
    return O.layer_rows(inp["X"], b, rows, inp["q"], inp["k"], inp["v"], inp["o"],
                        (inp["ln1_gamma"], inp["ln1_beta"]), inp["w1"], inp["w2"],
                        (inp["ln2_gamma"], inp["ln2_beta"]), w.H, norm=w.norm, causal=inp["causal"],
                        key_len=inp["key_len"], eps=w.ln_eps, part=part)


def gpu_call(dev, part="layer"):
    """The same computation through the C ABI; returns a float32 torch tensor on the device."""
    from paper_2508_01506_amd import binding as fb
    d = dev["desc"]
    if part == "attention":
        fn = fb.fsvd_attention_heads if isinstance(dev["q"], fb.HeadFactor) else fb.fsvd_attention
        return fn(d, dev["X"], dev["q"], dev["k"], dev["v"], dev["o"])
    if part == "ffn":
        return fb.fsvd_ffn(d, dev["X"], dev["w1"], dev["w2"])
    if part == "ffn_v2":
        return fb.fsvd_ffn_v2(d, dev["X"], dev["w1"], dev["w2"])
    fn = fb.fsvd_layer_heads if isinstance(dev["q"], fb.HeadFactor) else fb.fsvd_layer
    return fn(d, dev["X"], dev["q"], dev["k"], dev["v"], dev["o"], dev["ln1_gamma"], dev["ln1_beta"],
              dev["w1"], dev["w2"], dev["ln2_gamma"], dev["ln2_beta"])


def sample_rows(w: W.Workload, n_rows: int, seed: int = 0):
    """Sampled (sequence, rows) pairs: first and last rows, tile boundaries and random rows."""
    rng = np.random.default_rng(seed)
    fixed = [0, 1, 31, 32, 63, 64, 127, 128, 255, 256, 511, 512, w.M - 2, w.M - 1]
    rows = sorted({r for r in fixed if 0 <= r < w.M} | set(rng.integers(0, w.M, size=n_rows).tolist()))
    return rows
