"""Seeded synthetic workloads for the factored transformer layer.

This module only draws numbers and shapes them into the inputs of one layer
(activations X, rank-r factor pairs (U, V, b), LayerNorm parameters, key
lengths).  It contains none of the layer's arithmetic: no projection,
attention, activation or normalisation is evaluated here, so both the CPU
oracle's tests and the GPU path can consume exactly the same arrays.

Every array is generated in float64, cast to float32 and then rounded ONCE to
the 16-bit storage type of the workload (fp16 or bf16), so that the values a
GPU kernel reads from its 16-bit buffers and the values the oracle reads from
the float arrays are identical real numbers.

Factor format (Methodology, "Optimal Low-Rank Factorization via SVD"): a dense
projection W [in, out] is stored as U [in, r] and V [r, out] with the singular
values split evenly, U = A_r diag(sigma)^1/2, V = diag(sigma)^1/2 B_r^T, plus a
dense bias b [out].
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Optional

import numpy as np

__all__ = ["Workload", "WORKLOADS", "get_workload", "make_inputs", "round_to_storage",
           "to_storage_bits", "spectrum_factors", "DecodeWorkload", "DECODE_WORKLOADS", "make_decode_inputs"]


@dataclass(frozen=True)
class Workload:
    """Shape and recipe of one synthetic layer."""
    name: str
    B: int
    M: int
    D: int
    H: int
    F: int
    r_attn: int                 # rank of the four attention projections
    r_ffn: int                  # rank of the two FFN projections
    dtype: str                  # storage type of X and of every parameter: "fp16" | "bf16"
    mask: str = "none"          # "none" | "padding" | "causal"
    norm: str = "post_ln"       # "post_ln" | "pre_ln" | "none"
    factors: str = "gaussian"   # "gaussian" | "spectrum" | "spectrum_unit"
    min_len: int = 0            # padding mask: key_len ~ integers U[min_len, M]
    r_head: int = 0             # > 0: q, k, v are factored per head (or per head group) with this rank
                                # (U [D, G r], V [G, r, D / G]); the output projection keeps a whole-matrix
                                # factorisation of rank r_attn
    head_groups: int = 0        # with r_head > 0: number of head groups G sharing one factor pair (0 = one per head)
    seed: int = 1506
    ln_eps: float = 1e-5

    @property
    def T(self) -> int:
        return self.B * self.M

    @property
    def d_h(self) -> int:
        return self.D // self.H


def _wl(index: int, sub: int = 0, **kw) -> Workload:
    return Workload(seed=1506 + 1000 * index + sub, **kw)


# The five benchmark configurations plus small shapes used by the tests.
WORKLOADS: Dict[str, Workload] = {}


def _register(w: Workload) -> None:
    WORKLOADS[w.name] = w


_register(_wl(1, name="cfg1_bert_base_b2_m128", B=2, M=128, D=768, H=12, F=3072,
              r_attn=192, r_ffn=384, dtype="fp16"))
_register(_wl(2, name="cfg2_bert_base_b16_m512_pad", B=16, M=512, D=768, H=12, F=3072,
              r_attn=384, r_ffn=768, dtype="fp16", mask="padding", min_len=256,
              factors="spectrum"))
_register(_wl(2, 1, name="cfg2u_bert_base_b16_m512_pad_unit", B=16, M=512, D=768, H=12, F=3072,
              r_attn=384, r_ffn=768, dtype="fp16", mask="padding", min_len=256,
              factors="spectrum_unit"))
for _i, _r in enumerate((128, 256, 512)):
    _register(_wl(3, _i, name=f"cfg3_bert_large_b32_m512_r{_r}", B=32, M=512, D=1024, H=16,
                  F=4096, r_attn=_r, r_ffn=_r, dtype="bf16"))
_register(_wl(4, name="cfg4_long_b4_m8192", B=4, M=8192, D=768, H=12, F=3072,
              r_attn=256, r_ffn=512, dtype="fp16"))
_register(_wl(5, name="cfg5_llm_b1_m4096_causal", B=1, M=4096, D=4096, H=32, F=16384,
              r_attn=1024, r_ffn=2048, dtype="bf16", mask="causal", norm="pre_ln"))

# Small shapes: a few tiles plus ragged tails, cheap for the oracle.
_register(_wl(7, name="tiny_h2_d64", B=2, M=80, D=128, H=2, F=256, r_attn=48, r_ffn=80,
              dtype="fp16"))
_register(_wl(7, 1, name="tiny_pad", B=3, M=200, D=128, H=2, F=384, r_attn=64, r_ffn=96,
              dtype="fp16", mask="padding", min_len=1))
_register(_wl(7, 2, name="tiny_causal_d128", B=2, M=333, D=256, H=2, F=512, r_attn=80,
              r_ffn=144, dtype="bf16", mask="causal", norm="pre_ln"))
_register(_wl(7, 3, name="small_multi_qblock", B=2, M=1100, D=192, H=3, F=768, r_attn=96,
              r_ffn=208, dtype="fp16", mask="padding", min_len=300))
_register(_wl(7, 4, name="small_causal_d64", B=1, M=700, D=256, H=4, F=1024, r_attn=112,
              r_ffn=272, dtype="bf16", mask="causal", norm="none"))


# Widths 512 and 1024 at test size (the fused projection + LayerNorm kernel is specialised per D / 256).
# Widths 256..1024 with ragged token counts and small rank-by-width products: the shapes for which the last
# projection of a block, the residual add and the LayerNorm run as one kernel (prepacked weights, post-LN).
_register(_wl(7, 5, name="fuse_d512_pad", B=4, M=530, D=512, H=8, F=256, r_attn=80, r_ffn=96, dtype="bf16",
              mask="padding", min_len=40))
_register(_wl(7, 6, name="fuse_d1024", B=1, M=2100, D=1024, H=8, F=512, r_attn=64, r_ffn=112, dtype="fp16"))
_register(_wl(7, 7, name="fuse_d256_causal", B=3, M=700, D=256, H=4, F=512, r_attn=48, r_ffn=80, dtype="fp16",
              mask="causal"))
_register(_wl(7, 8, name="fuse_d768", B=2, M=1040, D=768, H=12, F=384, r_attn=96, r_ffn=64, dtype="bf16"))
# 16468 tokens = 514 full 32-token tiles and 20 rows: the one-kernel hand-off then runs 64 tokens per workgroup, the last
# workgroup holding a partial tile and a tile that does not exist.
_register(_wl(7, 14, name="fuse_wide_d256", B=4, M=4117, D=256, H=4, F=256, r_attn=48, r_ffn=64, dtype="fp16"))
_register(_wl(7, 15, name="fuse_wide_d512", B=2, M=8234, D=512, H=8, F=256, r_attn=64, r_ffn=96, dtype="bf16"))
_register(_wl(7, 16, name="fuse_wide_d1024", B=4, M=4117, D=1024, H=8, F=512, r_attn=64, r_ffn=80, dtype="bf16",
              mask="causal"))

# Shapes for the one-kernel FFN (FlashSVDFFN V2): ranks above 512 (two slabs of ranks), widths above 512 (two slabs of
# X and of the output), F that is not a multiple of the 128-, 256- or 512-wide units, ragged token counts, and enough
# tokens for the 64-token variant.
_register(_wl(7, 9, name="v2_two_rank_slabs", B=2, M=75, D=640, H=10, F=1104, r_attn=32, r_ffn=528, dtype="bf16"))
_register(_wl(7, 10, name="v2_max_rank", B=1, M=100, D=1024, H=8, F=2064, r_attn=32, r_ffn=1024, dtype="fp16"))
_register(_wl(7, 11, name="v2_many_tokens", B=26, M=500, D=128, H=2, F=400, r_attn=32, r_ffn=96, dtype="fp16"))
_register(_wl(7, 12, name="v2_many_tokens_r512", B=13, M=1001, D=576, H=9, F=784, r_attn=32, r_ffn=512, dtype="bf16"))
_register(_wl(7, 13, name="v2_llm_width_r1024", B=1, M=2048, D=4096, H=32, F=16384, r_attn=64, r_ffn=1024, dtype="bf16",
              norm="pre_ln"))

# Per-head factorisation of q, k, v (the paper's attention setting: one rank-r pair per head, r <= d_h), the encoder
# shapes of its attention-kernel sweep: batch 16 or 64, sequence 128..1024, per-head ranks 64, 32, 16.
for _i, (_b, _m, _r) in enumerate(((16, 512, 32), (16, 512, 64), (16, 512, 16), (64, 128, 32), (16, 1024, 48))):
    _register(_wl(8, _i, name=f"ph_bert_base_b{_b}_m{_m}_r{_r}", B=_b, M=_m, D=768, H=12, F=3072, r_attn=192,
                  r_ffn=384, dtype="fp16", mask="padding", min_len=_m // 2, r_head=_r))
_register(_wl(9, name="ph_tiny_r16", B=2, M=150, D=128, H=2, F=256, r_attn=48, r_ffn=64, dtype="fp16",
              mask="padding", min_len=1, r_head=16))
_register(_wl(9, 1, name="ph_tiny_r48_causal", B=2, M=300, D=192, H=3, F=384, r_attn=64, r_ffn=64, dtype="bf16",
              mask="causal", r_head=48))
_register(_wl(9, 2, name="ph_tiny_d128_r32", B=1, M=270, D=256, H=2, F=512, r_attn=80, r_ffn=64, dtype="bf16",
              r_head=32))
_register(_wl(9, 3, name="ph_tiny_d128_r64", B=2, M=200, D=256, H=2, F=512, r_attn=80, r_ffn=64, dtype="fp16",
              mask="padding", min_len=3, r_head=64))
_register(_wl(9, 4, name="ph_tiny_d128_r48_causal", B=1, M=330, D=384, H=3, F=512, r_attn=80, r_ffn=64, dtype="bf16",
              mask="causal", r_head=48))


# The paper's FFN rank ablation (table "Computation-efficiency ablation": batch 16, BERT-base widths, sequence
# 128 .. 1024, FFN ranks 768 / 384 / 192 / 96): the FFN block alone is of interest, the attention ranks are a filler.
FFN_GRID = [(m, r) for m in (128, 256, 512, 1024) for r in (768, 384, 192, 96)]
for _i, (_m, _r) in enumerate(FFN_GRID):
    _register(_wl(10, _i, name=f"ffn_grid_b16_m{_m}_r{_r}", B=16, M=_m, D=768, H=12, F=3072, r_attn=64, r_ffn=_r,
                  dtype="fp16"))


# Grouped heads (appendix, grouped-head compression): G groups of H / G heads share one rank-r pair per projection.
_register(_wl(11, name="gh_bert_base_b16_m512_g4_r96", B=16, M=512, D=768, H=12, F=3072, r_attn=192, r_ffn=384,
              dtype="fp16", mask="padding", min_len=256, r_head=96, head_groups=4))
_register(_wl(11, 1, name="gh_bert_base_b16_m512_g2_r192", B=16, M=512, D=768, H=12, F=3072, r_attn=192, r_ffn=384,
              dtype="fp16", mask="padding", min_len=256, r_head=192, head_groups=2))
_register(_wl(11, 2, name="gh_tiny_g2_r48_causal", B=2, M=150, D=256, H=4, F=256, r_attn=48, r_ffn=64, dtype="bf16",
              mask="causal", r_head=48, head_groups=2))
_register(_wl(11, 3, name="gh_tiny_d128_g2_r80", B=1, M=270, D=512, H=4, F=512, r_attn=80, r_ffn=64, dtype="fp16",
              mask="padding", min_len=100, r_head=80, head_groups=2))
_register(_wl(11, 4, name="gh_tiny_g1_r64", B=2, M=100, D=128, H=2, F=256, r_attn=48, r_ffn=64, dtype="fp16",
              r_head=64, head_groups=1))


def get_workload(name: str, **overrides) -> Workload:
    w = WORKLOADS[name]
    return replace(w, **overrides) if overrides else w


# ---------------------------------------------------------------------------
# rounding to the 16-bit storage types
# ---------------------------------------------------------------------------

def _bf16_bits(x32: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def to_storage_bits(x: np.ndarray, dtype: str) -> np.ndarray:
    """16-bit patterns (uint16 array) of ``x`` in storage type ``dtype``."""
    x32 = np.asarray(x, dtype=np.float32)
    if dtype == "fp16":
        return x32.astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        return _bf16_bits(x32)
    raise ValueError(f"unknown storage dtype {dtype!r}")


def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """``x`` rounded once to ``dtype`` and returned as float32 (exactly representable)."""
    x32 = np.asarray(x, dtype=np.float32)
    if dtype == "fp16":
        return x32.astype(np.float16).astype(np.float32)
    if dtype == "bf16":
        bits = _bf16_bits(x32).astype(np.uint32) << np.uint32(16)
        return bits.view(np.float32).reshape(x32.shape)
    if dtype == "fp32":
        return x32
    raise ValueError(f"unknown storage dtype {dtype!r}")


# ---------------------------------------------------------------------------
# factor generators
# ---------------------------------------------------------------------------

def _orthonormal(rng: np.random.Generator, rows: int, cols: int) -> np.ndarray:
    """Seeded matrix with orthonormal columns (QR of a Gaussian, signs fixed)."""
    q, r = np.linalg.qr(rng.standard_normal((rows, cols)))
    return q * np.sign(np.diag(r))[None, :]


def spectrum_factors(rng: np.random.Generator, n_in: int, n_out: int, rank: int,
                     unit: bool):
    """Rank-``rank`` truncation of W = A diag(sigma) B^T with sigma_i = c * i^-1/2.

    A [n_in, n], B [n_out, n] have orthonormal columns (n = min(n_in, n_out)),
    so the construction *is* the SVD of W and the best rank-r factors are known
    without calling an SVD routine.  ``unit`` chooses c so that X W has unit
    variance per element for X ~ N(0, 1) (c^2 = n_out / sum_i 1/i); otherwise c = 1.
    Returns (U, V, sigma) in float64, with sigma the full spectrum.
    """
    n = min(n_in, n_out)
    a = _orthonormal(rng, n_in, n)
    b = _orthonormal(rng, n_out, n)
    sigma = np.arange(1, n + 1, dtype=np.float64) ** -0.5
    if unit:
        sigma = sigma * np.sqrt(n_out / np.sum(1.0 / np.arange(1, n + 1)))
    root = np.sqrt(sigma[:rank])
    u = a[:, :rank] * root[None, :]
    v = root[:, None] * b[:, :rank].T
    return u, v, sigma


def _gaussian_factors(rng: np.random.Generator, n_in: int, n_out: int, rank: int):
    """U ~ N(0, 1/n_in), V ~ N(0, 1/rank): variance 1/fan_in of each factor."""
    u = rng.standard_normal((n_in, rank)) / np.sqrt(n_in)
    v = rng.standard_normal((rank, n_out)) / np.sqrt(rank)
    return u, v


def make_inputs(w: Workload) -> dict:
    """Draw every input of one layer for workload ``w``.

    Draw order: X; (U, V, b) for q, k, v, o; ln1 gamma, beta; (U, V, b) for
    w1, w2; ln2 gamma, beta; key_len.  Returns float32 arrays already rounded
    to ``w.dtype`` (key_len: int32 or None) and, for spectrum workloads, the
    float64 spectra under ``"sigma"``.
    """
    rng = np.random.Generator(np.random.PCG64(w.seed))
    st = w.dtype
    out: dict = {"workload": w}
    out["X"] = round_to_storage(rng.standard_normal((w.B, w.M, w.D)), st)

    sigma = {}

    def factor(name: str, n_in: int, n_out: int, rank: int):
        if w.factors == "gaussian":
            u, v = _gaussian_factors(rng, n_in, n_out, rank)
        else:
            u, v, s = spectrum_factors(rng, n_in, n_out, rank, unit=(w.factors == "spectrum_unit"))
            sigma[name] = s
        b = 0.02 * rng.standard_normal(n_out)
        out[name] = {"U": round_to_storage(u, st), "V": round_to_storage(v, st),
                     "b": round_to_storage(b, st)}

    def ln(name: str):
        out[name + "_gamma"] = round_to_storage(1.0 + 0.02 * rng.standard_normal(w.D), st)
        out[name + "_beta"] = round_to_storage(0.02 * rng.standard_normal(w.D), st)

    def head_factor(name: str):
        # per group (per head when G = H): U_g ~ N(0, 1/D) [D, r], V_g ~ N(0, 1/r) [r, D / G]; stored as U [D, G r]
        # (group g = columns g r ..) and V [G, r, D / G]
        r = w.r_head
        G = w.head_groups if w.head_groups > 0 else w.H
        u = rng.standard_normal((w.D, G * r)) / np.sqrt(w.D)
        v = rng.standard_normal((G, r, w.D // G)) / np.sqrt(r)
        b = 0.02 * rng.standard_normal(w.D)
        out[name] = {"U": round_to_storage(u, st), "V": round_to_storage(v, st), "b": round_to_storage(b, st)}

    for a in ("q", "k", "v", "o"):
        if w.r_head > 0 and a != "o":
            head_factor(a)
        else:
            factor(a, w.D, w.D, w.r_attn)
    ln("ln1")
    factor("w1", w.D, w.F, w.r_ffn)
    factor("w2", w.F, w.D, w.r_ffn)
    ln("ln2")
    if w.mask == "padding":
        out["key_len"] = rng.integers(max(w.min_len, 1), w.M + 1, size=w.B).astype(np.int32)
    else:
        out["key_len"] = None
    out["causal"] = (w.mask == "causal")
    if sigma:
        out["sigma"] = sigma
    return out


# ---------------------------------------------------------------------------
# decoding step against a rank-space KV cache
# ---------------------------------------------------------------------------

@dataclass(frozen=True)
class DecodeWorkload:
    """One decoding step: B sequences, each with its own number of cached tokens in [len_min, len_max] (< t_max)."""
    name: str
    B: int
    t_max: int
    D: int
    H: int
    r: int            # rank of q, k, v and o
    dtype: str        # storage of the new tokens and of the parameters
    len_min: int
    len_max: int
    seed: int

    @property
    def d_h(self) -> int:
        return self.D // self.H


DECODE_WORKLOADS = {w.name: w for w in [
    # the decoder shape of the largest prefill configuration (D 4096, 32 heads of 128, rank 1024), a batch of 16
    # sequences with 4096-token caches that are between half full and full
    DecodeWorkload("decode_llm_b16_t4096_r1024", 16, 4096, 4096, 32, 1024, "bf16", 2048, 4095, 7506),
    DecodeWorkload("decode_llm_b64_t2048_r512", 64, 2048, 4096, 32, 512, "bf16", 1024, 2047, 7507),
    DecodeWorkload("decode_base_b32_t1024_r256", 32, 1024, 768, 12, 256, "fp16", 1, 1023, 7508),
    DecodeWorkload("decode_tiny_d64", 3, 80, 128, 2, 64, "fp16", 0, 79, 7509),
    DecodeWorkload("decode_tiny_d128", 5, 300, 512, 4, 128, "bf16", 0, 299, 7510),
    DecodeWorkload("decode_tiny_b70", 70, 64, 128, 2, 64, "fp16", 0, 63, 7511),       # more than two sequence tiles
]}


def make_decode_inputs(w: DecodeWorkload) -> dict:
    """Seeded inputs of one decoding step.  Draw order: x_new; (U, V, b) for q, k, v, o (Gaussian, variance 1/fan_in);
    the cached rank-space keys and values (standard normal, the scale rank projections of unit-variance tokens have,
    rounded to fp16 as the cache stores them; rows at and beyond a sequence's length are drawn too and must be
    ignored); lens (the first and the last sequence get len_min and len_max)."""
    rng = np.random.Generator(np.random.PCG64(w.seed))
    st = w.dtype
    out: dict = {"workload": w, "x_new": round_to_storage(rng.standard_normal((w.B, w.D)), st)}
    for a in ("q", "k", "v", "o"):
        u, v = _gaussian_factors(rng, w.D, w.D, w.r)
        out[a] = {"U": round_to_storage(u, st), "V": round_to_storage(v, st),
                  "b": round_to_storage(0.02 * rng.standard_normal(w.D), st)}
    out["Pk"] = round_to_storage(rng.standard_normal((w.B, w.t_max, w.r), dtype=np.float32), "fp16")
    out["Pv"] = round_to_storage(rng.standard_normal((w.B, w.t_max, w.r), dtype=np.float32), "fp16")
    lens = rng.integers(w.len_min, w.len_max + 1, size=w.B).astype(np.int32)
    lens[0], lens[-1] = w.len_min, w.len_max
    out["lens"] = lens
    return out
