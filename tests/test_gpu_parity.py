"""Parity of the HIP path (through the C ABI) against the CPU oracle, element by element, on the
same seeded inputs.  Metric: max|err| / RMS(ref).

Tolerances.  The stated gate, 2e-3, is applied to fsvd_layer with a LayerNorm on every workload (measured on the
benchmark configurations: 1.1e-3 .. 1.8e-3).  The blocks called alone have no LayerNorm behind them and a smaller
output scale; tests/test_handoff_noise_model.py shows on the CPU which fp16 operand roundings produce their error and
that the unavoidable ones alone exceed 2e-3 for the attention block.  Their bounds are the values measured on the
benchmark configurations (whole sequences, reported by test_full_size_sampled_rows) plus a margin:
  * fsvd_ffn: three roundings (P1, activated hidden, Z) of about 1e-3 each at the maximum; measured 1.8e-3 .. 2.2e-3,
    and 3.3e-3 on the spectrum-built factors of the second configuration (a few dominant singular directions make the
    output heavier-tailed); bound 4e-3, and 3e-3 against each row's own RMS (measured <= 2.4e-3).
  * fsvd_attention, no mask / padding: measured 2.4e-3 .. 3.8e-3, and 7.9e-3 on the spectrum-built factors of the
    second configuration whose output RMS is 0.08; bound 1e-2, and 6e-3 for the same maximum taken against each
    row's own RMS (measured <= 4.4e-3).
  * fsvd_attention, causal: the first rows average one or a few keys and are O(1) next to an output RMS set by the
    many late rows; measured 1.24e-2 against the global RMS and 3.3e-3 against each row's own; bounds 2e-2 and 6e-3.
  * fsvd_layer with NORM_NONE (FFN(Attn(X)), nothing renormalises in between): 3e-2.
"""
import os

import dataclasses

import numpy as np
import pytest
import torch

from fsvd_testing import gpu_call, oracle_call, oracle_rows, rel_err, sample_rows
from oracle import fsvd_oracle as O
from paper_2508_01506_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL_LAYER = 2e-3
TOL = {"layer": TOL_LAYER, "ffn": 4e-3, "attention": 1e-2, "attention_causal": 2e-2, "layer_none": 3e-2}
TOL_PER_ROW = {"attention": 6e-3, "ffn": 3e-3}      # max|err| of a row over that row's own RMS


@pytest.fixture(scope="module")
def fb():
    from paper_2508_01506_amd import binding
    binding.lib()
    assert torch.cuda.is_available(), "these tests need the GPU"
    return binding


def tol_for(w, part):
    if part == "attention":
        return TOL["attention_causal"] if w.mask == "causal" else TOL["attention"]
    if part == "layer" and w.norm == "none":
        return TOL["layer_none"]
    return TOL[part]


DEV = "cuda:0"
_cache = {}


def workload(name, fb, weights="row"):
    """weights: "row" = factors as row-major tensors, "tiled" = the prepacked tile images wherever the library takes them."""
    key = (name, weights)
    if key not in _cache:
        if not any(k[0] == name for k in _cache):
            _cache.clear()
        inp = next((v[1] for k, v in _cache.items() if k[0] == name), None)
        if inp is None:
            inp = W.make_inputs(W.get_workload(name))
        _cache[key] = (inp["workload"], inp, fb.to_device(inp, DEV, tiled=(weights == "tiled")))
    return _cache[key]


WEIGHTS = ["row", "tiled"]


# ------------------------------------------------------------------ building blocks
@pytest.mark.parametrize("T,K,N,adt,wdt,odt", [
    (70, 64, 48, torch.float16, torch.float16, torch.float32),
    (300, 192, 272, torch.bfloat16, torch.bfloat16, torch.float32),
    (513, 208, 128, torch.float32, torch.float16, torch.float32),
    (256, 768, 576, torch.float16, torch.float16, torch.float16),
    (1, 16, 16, torch.float16, torch.float16, torch.float32),
    (1000, 1024, 80, torch.bfloat16, torch.bfloat16, torch.bfloat16),
    (2049, 2048, 3072, torch.float16, torch.bfloat16, torch.float32),
])
def test_linear(fb, T, K, N, adt, wdt, odt):
    g = torch.Generator().manual_seed(T + K + N)
    A = torch.randn(T, K, generator=g).to(adt)
    Wt = (torch.randn(K, N, generator=g) / K ** 0.5).to(wdt)
    b = torch.randn(N, generator=g).to(wdt)
    R = torch.randn(T, N, generator=g)
    # operands are exact in their storage type; an fp32 activation is rounded to fp16 by the kernel
    A_used = A.to(torch.float16) if adt == torch.float32 else A
    ref = O.rank_projection(A_used.double().numpy(), Wt.double().numpy()) + b.double().numpy() + R.double().numpy()
    got = fb.fsvd_linear(A.to(DEV), Wt.to(DEV), b.to(DEV), R.to(DEV), out_dtype=odt).float().cpu().numpy()
    out_eps = {torch.float32: 2e-6, torch.float16: 2.0 ** -11, torch.bfloat16: 2.0 ** -8}[odt]
    assert np.abs(got - ref).max() <= out_eps * (np.abs(ref).max() + 1) + 1e-5
    plain = fb.fsvd_linear(A.to(DEV), Wt.to(DEV), out_dtype=torch.float32).cpu().numpy()
    ref_plain = O.rank_projection(A_used.double().numpy(), Wt.double().numpy())
    assert rel_err(plain, ref_plain) < 5e-6


@pytest.mark.parametrize("T,K,N,adt,wdt", [(300, 96, 80, torch.float16, torch.float16), (513, 768, 1152, torch.bfloat16, torch.bfloat16),
                                           (64, 16, 16, torch.float32, torch.bfloat16), (1000, 1024, 200 * 16, torch.float32, torch.float16)])
def test_linear_with_tile_image_weights_matches_row_major(fb, T, K, N, adt, wdt):
    """The projections read prepacked weights in place of the row-major matrix: same values, same order of operations."""
    g = torch.Generator(device=DEV).manual_seed(T + N)
    A = torch.randn(T, K, generator=g, device=DEV).to(adt)
    Wm = (torch.randn(K, N, generator=g, device=DEV) * K ** -0.5).to(wdt)
    b = (0.1 * torch.randn(N, generator=g, device=DEV)).to(wdt)
    R = torch.randn(T, N, generator=g, device=DEV)
    want = fb.fsvd_linear(A, Wm, b, R, out_dtype=torch.float32)
    got = fb.fsvd_linear_tiled(A, fb.fsvd_pack_tiled(Wm), N, b, R, out_dtype=torch.float32)
    assert torch.equal(got, want)
    ref = A.double() @ Wm.double() + b.double() + R.double()
    assert rel_err(got.cpu().numpy(), ref.cpu().numpy()) < 2e-3


@pytest.mark.parametrize("T,D,xdt,ydt", [(37, 768, torch.float32, torch.float32), (5, 64, torch.float16, torch.float16),
                                         (130, 4096, torch.bfloat16, torch.float32), (3, 1104, torch.float32, torch.bfloat16)])
def test_layernorm(fb, T, D, xdt, ydt):
    g = torch.Generator().manual_seed(D)
    X = (torch.randn(T, D, generator=g) * 2 + 1).to(xdt)
    gm = torch.randn(D, generator=g).half()
    bt = torch.randn(D, generator=g).half()
    ref = O.layer_norm(X.double().numpy(), gm.double().numpy(), bt.double().numpy(), 1e-5)
    got = fb.fsvd_layernorm(X.to(DEV), gm.to(DEV), bt.to(DEV), 1e-5, out_dtype=ydt).float().cpu().numpy()
    eps = {torch.float32: 3e-6, torch.float16: 2.0 ** -11, torch.bfloat16: 2.0 ** -8}[ydt]
    assert np.abs(got - ref).max() <= eps * (np.abs(ref).max() + 1)


@pytest.mark.parametrize("T,K,dt", [(70, 48, torch.float16), (257, 208, torch.bfloat16), (64, 64, torch.float32), (1, 16, torch.float16)])
def test_fragment_major_pack_unpack_roundtrip(fb, T, K, dt):
    """pack places element (t, k) where the documented layout says, zero-fills the padding, and unpack inverts it."""
    g = torch.Generator().manual_seed(T * K)
    A = torch.randn(T, K, generator=g).to(dt)
    fm = fb.fsvd_pack_fm(A.to(DEV))
    assert fm.numel() == ((T + 31) // 32) * ((K + 63) // 64) * 4096
    halves = fm.cpu().view(torch.float16).numpy()
    ref = np.zeros_like(halves)
    A16 = A.to(torch.float16).numpy()
    kc = (K + 63) // 64
    for t in range(T):
        for k in range(K):
            c, gg, kk, s = k // 64, (k // 32) % 2, (k // 8) % 4, k % 8
            unit = (((t // 32) * kc + c) * 4 + kk) * 64 + gg * 32 + t % 32
            ref[unit * 8 + s] = A16[t, k]
    np.testing.assert_array_equal(halves, ref)
    back = fb.fsvd_unpack_fm(fm, T, K, torch.float32).cpu().numpy()
    np.testing.assert_array_equal(back, A16.astype(np.float32))


def _selector(total, start, width):
    S = np.zeros((total, width))
    S[np.arange(start, start + width), np.arange(width)] = 1.0
    return S


@pytest.mark.parametrize("name", ["tiny_h2_d64", "tiny_pad", "tiny_causal_d128", "small_multi_qblock"])
def test_attention_core_from_rank_space_inputs(fb, name):
    """Alg. 1 Part II alone: P_q, P_k, P_v (already fp16) -> context, against the oracle fed the same P."""
    w, inp, dev = workload(name, fb)
    r = w.r_attn
    P = {a: O.rank_projection(inp["X"], inp[a]["U"]).astype(np.float16) for a in "qkv"}
    Pd = {a: fb.fsvd_pack_fm(torch.from_numpy(P[a].reshape(w.T, r)).to(DEV)) for a in "qkv"}
    ctx = fb.fsvd_attention_core(dev["desc"], Pd["q"], Pd["k"], Pd["v"], dev["q"], dev["k"], dev["v"])
    got = fb.fsvd_unpack_fm(ctx, w.T, w.D, torch.float32).cpu().numpy().reshape(w.B, w.M, w.D)
    # oracle on x = [P_q | P_k | P_v] with 0/1 selector matrices as the U factors
    xcat = np.concatenate([P[a].astype(np.float64) for a in "qkv"], axis=-1)
    fac = {a: {"U": _selector(3 * r, i * r, r), "V": inp[a]["V"], "b": inp[a]["b"]} for i, a in enumerate("qkv")}
    ref = np.stack([O.attention_context_one_sequence(xcat[b], fac["q"], fac["k"], fac["v"], w.H, inp["causal"],
                                                     None if inp["key_len"] is None else inp["key_len"][b])
                    for b in range(w.B)])
    # hand-offs left: Q/K/V tiles, probabilities, and the fp16 context itself, whose final rounding is
    # not averaged by any later contraction (half an ulp of a 4.5-sigma element is 2.2e-3 of the RMS)
    assert rel_err(got, ref) < (2e-2 if inp["causal"] else 8e-3)


def expected_tile_images(Wm):
    """The documented byte image of a weight matrix (fp16 values), written from the format's definition."""
    K, N = Wm.shape
    kt, nt = (K + 127) // 128, (N + 127) // 128
    pad = np.zeros((kt * 128, nt * 128), np.float16)
    pad[:K, :N] = Wm
    out = np.empty((kt, nt, 128, 128), np.float16)
    for k in range(128):
        for seg in range(4):
            out[:, :, k, 32 * (seg ^ (k & 3)):32 * (seg ^ (k & 3)) + 32] = \
                pad.reshape(kt, 128, nt, 128)[:, k, :, 32 * seg:32 * seg + 32]
    return out.reshape(-1)


@pytest.mark.parametrize("K,N,dt", [(256, 1024, "fp16"), (200, 336, "bf16"), (16, 16, "fp16"), (1040, 136, "bf16"), (128, 128, "fp16")])
def test_pack_tiled_writes_the_documented_image(fb, K, N, dt):
    """Byte work: the prepacked tile images are bit-exact (values inside fp16's normal range, where widening bf16
    is exact; ragged edges are zero-padded to whole tiles)."""
    rng = np.random.default_rng(K + N)
    x = rng.standard_normal((K, N)).astype(np.float32)
    Wm = W.round_to_storage(np.where(np.abs(x) < 1e-3, np.float32(1e-3), x), dt)
    tdt = torch.float16 if dt == "fp16" else torch.bfloat16
    src = torch.from_numpy(Wm).to(device=DEV, dtype=tdt).contiguous()
    assert fb.fsvd_tiled_bytes(K, N) == ((K + 127) // 128) * ((N + 127) // 128) * 32768
    img = fb.fsvd_pack_tiled(src).view(torch.float16).cpu().numpy()
    assert np.array_equal(img.view(np.uint16), expected_tile_images(Wm.astype(np.float16)).view(np.uint16))


@pytest.mark.parametrize("name,act", [("tiny_h2_d64", "gelu_erf"), ("tiny_pad", "gelu_tanh"), ("tiny_causal_d128", "relu"),
                                      ("small_causal_d64", "gelu_erf")])
def test_ffn_core_from_rank_space_input(fb, name, act):
    """The on-chip loops of Alg. 2 alone: P1 (fp16) -> Z = phi(P1 V_1 + b_1) U_2."""
    w, inp, dev = workload(name, fb)
    P1 = O.rank_projection(inp["X"], inp["w1"]["U"]).astype(np.float16).reshape(w.T, w.r_ffn)
    d = fb.make_desc(w.B, w.M, w.D, w.H, w.F, dev["X"].dtype, act=act)
    Zfm = fb.fsvd_ffn_core(d, fb.fsvd_pack_fm(torch.from_numpy(P1).to(DEV)), dev["w1"], dev["w2"])
    got = fb.fsvd_unpack_fm(Zfm, w.T, w.r_ffn, torch.float32).cpu().numpy()
    hidden = O.activation(P1.astype(np.float64) @ inp["w1"]["V"].astype(np.float64) + inp["w1"]["b"], act)
    ref = O.rank_projection(hidden, inp["w2"]["U"])
    assert rel_err(got, ref) < 2.5e-3      # fp16 hidden activation + fp16 Z


@pytest.mark.parametrize("weights", WEIGHTS)
@pytest.mark.parametrize("r2,dt", [(1024, "fp16"), (1024, "bf16"), (896, "fp16"), (640, "bf16")])
def test_ffn_core_wide_rank_slices_and_split_over_f(fb, r2, dt, weights):
    """Shapes for which the core lets one workgroup cover more than 512 output ranks (the extra accumulators live in
    the loader wavefronts) and splits the sum over D_ff across workgroups (fp32 partial sums + a second launch):
    sampled rows of Z against the plain definition, ragged token count, tanh-free exact GELU."""
    T, D, F, r1 = 8192 - 37, 128, 8192, 256
    rng = np.random.default_rng(77 + r2)
    tdt = torch.float16 if dt == "fp16" else torch.bfloat16
    rnd = lambda a: W.round_to_storage(a.astype(np.float32), dt).astype(np.float64)
    V1 = rnd(rng.standard_normal((r1, F)) / np.sqrt(r1))
    b1 = rnd(0.02 * rng.standard_normal(F))
    U2 = rnd(rng.standard_normal((F, r2)) / np.sqrt(F))
    P1 = rng.standard_normal((T, r1)).astype(np.float16)
    up = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float32)).to(device=DEV, dtype=tdt).contiguous()
    # U of w1 and V of w2 are not read by the core: any tensors of the right shape do
    w1 = fb.Factor(up(np.zeros((D, r1))), up(V1), up(b1))
    w2 = fb.Factor(up(U2), up(np.zeros((r2, D))), None)
    if weights == "tiled":
        w1, w2 = w1.with_tiled(v=True), w2.with_tiled(u=True)
    d = fb.make_desc(1, T, D, 2, F, tdt)
    assert fb.fsvd_ffn_core_workspace(d, r1, r2) > 0          # this shape does split F
    Zfm = fb.fsvd_ffn_core(d, fb.fsvd_pack_fm(torch.from_numpy(P1).to(DEV)), w1, w2)
    got = fb.fsvd_unpack_fm(Zfm, T, r2, torch.float32).cpu().numpy()
    rows = np.unique(np.concatenate([np.arange(0, 70), np.arange(T - 70, T), rng.integers(0, T, 200)]))
    hidden = O.activation(P1[rows].astype(np.float64) @ V1 + b1, "gelu_erf")
    ref = hidden @ U2
    assert np.isfinite(got).all()
    assert rel_err(got[rows], ref) < 2.5e-3
    again = fb.fsvd_unpack_fm(fb.fsvd_ffn_core(d, fb.fsvd_pack_fm(torch.from_numpy(P1).to(DEV)), w1, w2), T, r2,
                              torch.float32).cpu().numpy()
    assert np.array_equal(got, again)                          # partial sums are added in a fixed order


@pytest.mark.parametrize("name", ["tiny_h2_d64", "tiny_pad", "tiny_causal_d128", "small_multi_qblock", "small_causal_d64",
                                  "cfg1_bert_base_b2_m128", "fuse_d768"])
def test_ffn_all_wavefront_core_forced_on_small_and_ragged_shapes(fb, name, monkeypatch):
    """The all-wavefront FFN core is chosen by default only for output ranks >= 1024; FSVD_FFN_CORE=wide forces it so
    that its edge handling is covered too: token counts that are not multiples of 64, F below and not a multiple of the
    256-feature chunk, ranks of 16..768 (one to three 256-rank groups, partly empty), F split across workgroups: every
    element of the FFN block against the oracle, and bitwise repeatable."""
    monkeypatch.setenv("FSVD_FFN_CORE", "wide")
    w, inp, dev = workload(name, fb, "tiled")
    got = gpu_call(dev, "ffn")
    assert torch.isfinite(got).all()
    err = rel_err(got.cpu().numpy(), oracle_call(inp, "ffn"))
    _report(f"PARITY {name} weights=tiled part=ffn (all-wavefront core forced) max_err_over_rms={err:.3e}")
    assert err < tol_for(w, "ffn")
    assert torch.equal(got, gpu_call(dev, "ffn"))
    monkeypatch.setenv("FSVD_FFN_CORE", "tworole")
    other = gpu_call(dev, "ffn")
    assert rel_err(other.cpu().numpy(), got.cpu().numpy()) < 3e-3   # same function, other summation order: both round independently


# ------------------------------------------------------------------ per-head factors of q, k, v
def attn_block_tol(w, ref):
    """Tolerance of an attention block called alone: the derived relative bound for RMS(ref) >= 0.2, and for outputs
    of smaller scale (short unmasked sequences with low per-head ranks average the values down) the same absolute
    fp16 hand-off noise, 1e-3 at the maximum, expressed relative to RMS(ref)."""
    return max(tol_for(w, "attention"), 1.0e-3 / float(np.sqrt(np.mean(np.asarray(ref, dtype=np.float64) ** 2))))


@pytest.mark.parametrize("weights", WEIGHTS)
@pytest.mark.parametrize("name", ["ph_tiny_r16", "ph_tiny_r48_causal", "ph_tiny_d128_r32", "ph_tiny_d128_r64",
                                  "ph_tiny_d128_r48_causal"])
def test_attention_with_per_head_factors_small(fb, name, weights):
    """Every element of the attention block with per-head factors (ranks 16, 48 - which straddles the 64-rank
    chunks - and 32, 48, 64 with 128-wide heads) against the per-head oracle."""
    w, inp, dev = workload(name, fb, weights)
    got = gpu_call(dev, "attention").cpu().numpy()
    assert np.isfinite(got).all()
    ref = oracle_call(inp, "attention")
    assert rel_err(got, ref) < attn_block_tol(w, ref)


@pytest.mark.parametrize("name", ["ph_bert_base_b16_m512_r32", "ph_bert_base_b16_m512_r64", "ph_bert_base_b16_m512_r16",
                                  "ph_bert_base_b64_m128_r32", "ph_bert_base_b16_m1024_r48"])
def test_attention_with_per_head_factors_encoder_shapes(fb, name):
    """The encoder shapes of the paper's attention-kernel sweep, whole sequences against the per-head oracle."""
    w, inp, dev = workload(name, fb)
    got = gpu_call(dev, "attention").cpu().numpy()
    assert np.isfinite(got).all()
    for b in (0, w.B // 2, w.B - 1):
        one = dict(inp, X=inp["X"][b:b + 1], key_len=None if inp["key_len"] is None else inp["key_len"][b:b + 1])
        ref = oracle_call(one, "attention")
        assert rel_err(got[b:b + 1], ref) < attn_block_tol(w, ref)


@pytest.mark.parametrize("name", ["gh_tiny_g2_r48_causal", "gh_tiny_d128_g2_r80", "gh_tiny_g1_r64"])
def test_attention_and_layer_with_grouped_head_factors_small(fb, name):
    """Grouped heads (G groups of H / G heads share one factor pair): every element of the block and of the layer; the
    group's rank window straddles 64-rank chunks (48, 80), both head widths, G = 1 included."""
    w, inp, dev = workload(name, fb)
    got = gpu_call(dev, "attention").cpu().numpy()
    ref = oracle_call(inp, "attention")
    assert np.isfinite(got).all()
    assert rel_err(got, ref) < attn_block_tol(w, ref)
    assert rel_err(gpu_call(dev, "layer").cpu().numpy(), oracle_call(inp, "layer")) < TOL_LAYER


def test_one_group_of_all_heads_equals_the_whole_matrix_block(fb):
    """G = 1 is the whole-matrix factorisation: the grouped entry point must agree with fsvd_attention on the same factors."""
    w, inp, dev = workload("gh_tiny_g1_r64", fb)
    whole = {n: fb.Factor(dev[n].U, dev[n].V[0].contiguous(), dev[n].b) for n in "qkv"}
    a = fb.fsvd_attention_heads(dev["desc"], dev["X"], dev["q"], dev["k"], dev["v"], dev["o"])
    b = fb.fsvd_attention(dev["desc"], dev["X"], whole["q"], whole["k"], whole["v"], dev["o"])
    assert torch.equal(a, b)


@pytest.mark.parametrize("name", ["gh_bert_base_b16_m512_g4_r96", "gh_bert_base_b16_m512_g2_r192"])
def test_layer_with_grouped_head_factors_encoder_shapes(fb, name):
    w, inp, dev = workload(name, fb, "tiled")
    got = gpu_call(dev, "layer").cpu().numpy()
    for b in (0, w.B - 1):
        one = dict(inp, X=inp["X"][b:b + 1], key_len=None if inp["key_len"] is None else inp["key_len"][b:b + 1])
        assert rel_err(got[b:b + 1], oracle_call(one, "layer")) < TOL_LAYER


def test_absorbed_and_rebuilding_schedules_agree_on_seeded_random_shapes(fb, monkeypatch):
    """A sweep of seeded shapes (head count, head width, per-head rank, sequence length, mask, storage type) through both
    schedules of the per-head core: the rank windows then straddle the 64-rank chunks of the concatenated axis in every
    possible way and the sequences end at every position of a key tile and a key step.  The two kernels share no code
    after the rank projections, so their agreement to the hand-off noise of two blocks is a check of both; every fourth
    shape is also compared with the oracle."""
    rng = np.random.default_rng(20250801)
    for case in range(16):
        d_h = int(rng.choice([64, 128]))
        H = int(rng.integers(1, 7))
        r = int(rng.choice([16, 32, 48, 64]))
        M = int(rng.integers(1, 420))
        B = int(rng.integers(1, 4))
        mask = str(rng.choice(["none", "padding", "causal"]))
        dtype = str(rng.choice(["fp16", "bf16"]))
        w = W.Workload(name=f"sweep{case}", seed=9000 + case, B=B, M=M, D=H * d_h, H=H, F=2 * H * d_h, r_attn=32, r_ffn=32,
                       dtype=dtype, mask=mask, min_len=1, r_head=r)
        inp = W.make_inputs(w)
        dev = fb.to_device(inp, DEV)
        absorbed = gpu_call(dev, "attention").cpu().numpy()
        monkeypatch.setenv("FSVD_ATTN_ABSORBED", "0")
        rebuilt = gpu_call(dev, "attention").cpu().numpy()
        monkeypatch.delenv("FSVD_ATTN_ABSORBED")
        tag = (case, H, d_h, r, B, M, mask, dtype)
        assert np.isfinite(absorbed).all() and np.isfinite(rebuilt).all(), tag
        rms = float(np.sqrt(np.mean(rebuilt.astype(np.float64) ** 2)))
        tol = 1.5 * max(TOL["attention_causal" if mask == "causal" else "attention"], 1.0e-3 / rms)
        assert rel_err(absorbed, rebuilt) < tol, tag
        if case % 4 == 0:
            ref = oracle_call(inp, "attention")
            assert rel_err(absorbed, ref) < max(attn_block_tol(w, ref), TOL["attention_causal"] if mask == "causal" else 0.0), tag


@pytest.mark.parametrize("ranks", [(32, 16, 48), (16, 64, 32), (64, 48, 16)])
@pytest.mark.parametrize("name", ["ph_tiny_d128_r64", "ph_bert_base_b16_m512_r64"])
def test_per_head_factors_with_three_different_ranks(fb, name, ranks):
    """r_q, r_k and r_v differ (the first ranks of every head's pair are kept): the rank windows of the three
    projections then lie at different places of their concatenated axes."""
    w, inp, _ = workload(name, fb)
    inp = dict(inp)
    if w.B > 2:
        inp["X"] = inp["X"][:2]
        inp["key_len"] = None if inp["key_len"] is None else inp["key_len"][:2]
        w = dataclasses.replace(w, B=2)
        inp["workload"] = w
    for nm, r in zip("qkv", ranks):
        f = inp[nm]
        H, r0, d_h = f["V"].shape
        inp[nm] = {"U": np.ascontiguousarray(f["U"].reshape(w.D, H, r0)[:, :, :r].reshape(w.D, H * r)),
                   "V": np.ascontiguousarray(f["V"][:, :r]), "b": f["b"]}
    dev = fb.to_device(inp, DEV)
    got = gpu_call(dev, "attention").cpu().numpy()
    ref = oracle_call(inp, "attention")
    assert np.isfinite(got).all()
    assert rel_err(got, ref) < attn_block_tol(w, ref)
    assert rel_err(gpu_call(dev, "layer").cpu().numpy(), oracle_call(inp, "layer")) < TOL_LAYER


@pytest.mark.parametrize("norm", ["post_ln", "pre_ln"])
@pytest.mark.parametrize("name", ["ph_tiny_r16", "ph_tiny_r48_causal", "ph_tiny_d128_r32", "ph_tiny_d128_r64",
                                  "ph_tiny_d128_r48_causal"])
def test_layer_with_per_head_attention_meets_the_gate(fb, name, norm):
    w = W.get_workload(name, norm=norm)
    inp = W.make_inputs(w)
    dev = fb.to_device(inp, DEV)
    assert rel_err(gpu_call(dev, "layer").cpu().numpy(), oracle_call(inp, "layer")) < TOL_LAYER


@pytest.mark.parametrize("weights", WEIGHTS)
@pytest.mark.parametrize("name", ["ph_bert_base_b16_m512_r32", "ph_bert_base_b16_m1024_r48"])
def test_layer_with_per_head_attention_encoder_shapes(fb, name, weights):
    w, inp, dev = workload(name, fb, weights)
    got = gpu_call(dev, "layer").cpu().numpy()
    for b in (0, w.B - 1):
        one = dict(inp, X=inp["X"][b:b + 1], key_len=None if inp["key_len"] is None else inp["key_len"][b:b + 1])
        assert rel_err(got[b:b + 1], oracle_call(one, "layer")) < TOL_LAYER


def test_per_head_factors_agree_with_block_diagonal_whole_matrix_factors(fb, monkeypatch):
    """The same projections written as whole-matrix factors (V block diagonal) go through fsvd_attention.  With the
    rebuilding schedule forced, both entry points must agree to rounding (they differ only in how many zero ranks the
    rebuild multiplies); the absorbed schedule, which per-head ranks <= 64 take by default, rounds other intermediates
    (M_h, w_h and u_h instead of q, K and V), so it agrees with the rebuilding one to two blocks' worth of hand-off
    noise and with the oracle to the block's tolerance."""
    w, inp, dev = workload("ph_tiny_r16", fb)
    H, r, d_h = inp["q"]["V"].shape
    def whole(f):
        V = np.zeros((H * r, w.D), dtype=np.float32)
        for h in range(H):
            V[h * r:(h + 1) * r, h * d_h:(h + 1) * d_h] = f["V"][h]
        up = lambda a: torch.from_numpy(a).to(device=DEV, dtype=dev["X"].dtype).contiguous()
        return fb.Factor(up(f["U"]), up(V), up(f["b"]))
    same = fb.fsvd_attention(dev["desc"], dev["X"], whole(inp["q"]), whole(inp["k"]), whole(inp["v"]), dev["o"]).cpu().numpy()
    absorbed = gpu_call(dev, "attention").cpu().numpy()
    monkeypatch.setenv("FSVD_ATTN_ABSORBED", "0")
    rebuilt = gpu_call(dev, "attention").cpu().numpy()
    monkeypatch.delenv("FSVD_ATTN_ABSORBED")
    assert rel_err(rebuilt, same) < 1e-3
    assert not np.array_equal(absorbed, rebuilt)          # the switch really selects another kernel
    assert rel_err(absorbed, rebuilt) < 1.5 * TOL["attention"]


@pytest.mark.parametrize("name", ["ph_tiny_r16", "ph_tiny_r48_causal", "ph_tiny_d128_r32", "ph_bert_base_b16_m512_r32",
                                  "ph_bert_base_b16_m1024_r48"])
def test_rebuilding_schedule_still_serves_per_head_factors(fb, name, monkeypatch):
    """Per-head ranks <= 64 take the absorbed schedule by default; the rebuilding kernel stays reachable through
    FSVD_ATTN_ABSORBED=0 and must meet the same bars (block tolerance, layer gate)."""
    monkeypatch.setenv("FSVD_ATTN_ABSORBED", "0")
    w, inp, dev = workload(name, fb)
    got = gpu_call(dev, "attention").cpu().numpy()
    lay = gpu_call(dev, "layer").cpu().numpy()
    for b in sorted({0, w.B - 1}):
        one = dict(inp, X=inp["X"][b:b + 1], key_len=None if inp["key_len"] is None else inp["key_len"][b:b + 1])
        ref = oracle_call(one, "attention")
        assert rel_err(got[b:b + 1], ref) < attn_block_tol(w, ref)
        assert rel_err(lay[b:b + 1], oracle_call(one, "layer")) < TOL_LAYER


# ------------------------------------------------------------------ entry points, small shapes, every element
SMALL = ["tiny_h2_d64", "tiny_pad", "tiny_causal_d128", "small_multi_qblock", "small_causal_d64"]


@pytest.mark.parametrize("weights", WEIGHTS)
@pytest.mark.parametrize("part", ["attention", "ffn", "layer"])
@pytest.mark.parametrize("name", SMALL)
def test_entry_points_small(fb, name, part, weights):
    w, inp, dev = workload(name, fb, weights)
    got = gpu_call(dev, part).cpu().numpy()
    assert np.isfinite(got).all()
    assert rel_err(got, oracle_call(inp, part)) < tol_for(w, part)


@pytest.mark.parametrize("norm", ["post_ln", "pre_ln"])
@pytest.mark.parametrize("name", SMALL)
def test_layer_gate_on_small_shapes_both_norms(fb, name, norm):
    w = W.get_workload(name, norm=norm)
    inp = W.make_inputs(w)
    dev = fb.to_device(inp, DEV)
    assert rel_err(gpu_call(dev, "layer").cpu().numpy(), oracle_call(inp, "layer")) < TOL_LAYER


@pytest.mark.parametrize("name", ["fuse_d256_causal", "fuse_d512_pad", "fuse_d768", "fuse_d1024", "cfg1_bert_base_b2_m128"])
def test_post_ln_layer_with_projection_and_layernorm_fused(fb, name):
    """Post-LN layers of width 256, 512, 768 or 1024 with at least 256 tokens and a moderate rank-by-width product run the
    last projection of each block, the residual add and the LayerNorm as one kernel when the weights are prepacked:
    every element against the oracle, and the same layer with row-major weights (separate projection and LayerNorm
    kernels) for comparison; ragged token counts.  The last case has exactly 256 tokens."""
    w = W.get_workload(name, norm="post_ln")
    inp = W.make_inputs(w)
    ref = oracle_call(inp, "layer")
    fused = gpu_call(fb.to_device(inp, DEV, tiled=True), "layer").cpu().numpy()
    plain = gpu_call(fb.to_device(inp, DEV), "layer").cpu().numpy()
    assert np.isfinite(fused).all()
    assert rel_err(fused, ref) < TOL_LAYER
    assert rel_err(plain, ref) < TOL_LAYER
    # same arithmetic up to the order of the fp32 row statistics; one unit in the fp16 rounding of an intermediate is 1e-3
    assert rel_err(fused, plain) < TOL_LAYER


@pytest.mark.parametrize("name", ["fuse_wide_d256", "fuse_wide_d512", "fuse_wide_d1024"])
def test_fused_projection_and_layernorm_with_64_token_workgroups(fb, name):
    """From 16384 tokens on the fused kernel takes 64 tokens per workgroup: 16468 tokens (an odd number of 32-token
    tiles, the last one partial), sampled rows of the first and last sequence including the very last rows."""
    w, inp, dev = workload(name, fb, "tiled")
    assert w.B * w.M == 16468
    got = gpu_call(dev, "layer").cpu().numpy()
    assert np.isfinite(got).all()
    for b in (0, w.B - 1):
        rows = sample_rows(w, 12, seed=b)
        ref = oracle_rows(inp, b, rows, "layer")
        assert rel_err(got[b, rows], ref) < TOL_LAYER, (name, b)


# ------------------------------------------------------------------ benchmark sizes, sampled rows
FULL = ["cfg1_bert_base_b2_m128", "cfg2_bert_base_b16_m512_pad", "cfg2u_bert_base_b16_m512_pad_unit",
        "cfg3_bert_large_b32_m512_r128", "cfg3_bert_large_b32_m512_r256", "cfg3_bert_large_b32_m512_r512",
        "cfg4_long_b4_m8192", "cfg5_llm_b1_m4096_causal"]


_oracle_cache = {}


def _report(line):
    """Measured errors go to stdout (pytest -s) and, on a box that has the folder, to gpurun_out/parity_errors.txt."""
    print(line, flush=True)
    out_dir = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out")
    if os.path.isdir(out_dir):
        with open(os.path.join(out_dir, "parity_errors.txt"), "a") as f:
            f.write(line + "\n")


def _full_size_reference(name, inp, w):
    """Oracle rows for one benchmark workload: every row of sequences of up to 512 tokens, 200 rows (tile boundaries,
    first and last rows, random rows) of longer ones; first, middle and last sequence.  Cached: both weight layouts
    compare against the same reference."""
    if name not in _oracle_cache:
        ref = {}
        for b in sorted({0, w.B // 2, w.B - 1}):
            rows = list(range(w.M)) if w.M <= 512 else sample_rows(w, 200, seed=b)
            ref[b] = (rows, {part: oracle_rows(inp, b, rows, part) for part in ("layer", "attention", "ffn")})
        _oracle_cache.clear()
        _oracle_cache[name] = ref
    return _oracle_cache[name]


@pytest.mark.parametrize("weights", WEIGHTS)
@pytest.mark.parametrize("name", FULL)
def test_full_size_sampled_rows(fb, name, weights):
    """At the benchmark sizes, in the launch configuration bench.py times (prepacked weights; and with row-major
    weights), on rows the oracle computes one by one: whole sequences where they have at most 512 tokens, 200 rows per
    sequence otherwise.  The measured errors of the layer and of the two blocks called alone are reported."""
    w, inp, dev = workload(name, fb, weights)
    outs = {part: gpu_call(dev, part).cpu().numpy() for part in ("layer", "attention", "ffn")}
    ref = _full_size_reference(name, inp, w)
    for part, got in outs.items():
        assert np.isfinite(got).all()
        num, den, cnt, row_rel = 0.0, 0.0, 0, 0.0
        for b, (rows, r) in ref.items():
            diff = np.abs(got[b, rows] - r[part])
            num = max(num, float(diff.max()))
            den += float(np.sum(r[part] ** 2))
            cnt += r[part].size
            # the same maximum measured against each row's own RMS (rows of very different scale, e.g. under a causal mask)
            row_rel = max(row_rel, float((diff.max(axis=-1) / np.sqrt(np.mean(r[part] ** 2, axis=-1))).max()))
        rms = np.sqrt(den / cnt)
        err = num / rms
        _report(f"PARITY {name} weights={weights} part={part} rows={cnt // w.D} max_err_over_rms={err:.3e} "
                f"rms_ref={rms:.3e} max_err_over_row_rms={row_rel:.3e}")
        assert err < tol_for(w, part), (name, part, err)
        if part in TOL_PER_ROW:
            assert row_rel < TOL_PER_ROW[part], (name, part, row_rel)


def test_largest_configuration_every_row_of_the_layer(fb):
    """The decoder-shaped configuration in the form the benchmark times (prepacked weights, pre-LN, causal): all 4096
    rows of fsvd_layer against the oracle, at the stated 2e-3."""
    name = "cfg5_llm_b1_m4096_causal"
    w, inp, dev = workload(name, fb, "tiled")
    got = gpu_call(dev, "layer").cpu().numpy()
    assert np.isfinite(got).all()
    ref = oracle_call(inp, "layer")
    err = rel_err(got, ref)
    _report(f"PARITY {name} weights=tiled part=layer rows={w.T} (all) max_err_over_rms={err:.3e}")
    assert err < TOL_LAYER, err


@pytest.mark.parametrize("m,r", W.FFN_GRID)
def test_ffn_block_on_the_rank_ablation_grid(fb, m, r):
    """The FFN block (Alg. 2 with its two plain projections) on the sequence lengths and ranks of the paper's FFN rank
    ablation, prepacked weights, sampled rows against the oracle."""
    w, inp, dev = workload(f"ffn_grid_b16_m{m}_r{r}", fb, "tiled")
    got = gpu_call(dev, "ffn").cpu().numpy()
    assert np.isfinite(got).all()
    for b in (0, w.B - 1):
        rows = sample_rows(w, 10, seed=b)
        assert rel_err(got[b, rows], oracle_rows(inp, b, rows, "ffn")) < tol_for(w, "ffn"), (m, r, b)


V2_SMALL = SMALL + ["v2_two_rank_slabs", "v2_max_rank", "v2_many_tokens", "v2_many_tokens_r512", "fuse_d768"]


@pytest.mark.parametrize("name", V2_SMALL)
def test_ffn_as_one_kernel_small(fb, name):
    """FlashSVDFFN V2 (Alg. 3): X -> out in one kernel without workspace, every element against the oracle's FFN and
    against the V1 entry point (the same fp16 hand-offs)."""
    w, inp, dev = workload(name, fb, "tiled")
    got = gpu_call(dev, "ffn_v2").cpu().numpy()
    assert np.isfinite(got).all()
    err = rel_err(got, oracle_call(inp, "ffn"))
    assert err < tol_for(w, "ffn")
    # the two kernels sum in different orders, so their fp16 hand-offs round differently here and there
    err_v1 = rel_err(got, gpu_call(dev, "ffn").cpu().numpy())
    assert err_v1 < 3e-3


@pytest.mark.parametrize("T,D,F,r1,r2,dt", [
    (1, 64, 16, 16, 16, torch.float16),             # one token, one step of everything
    (33, 64, 48, 32, 16, torch.bfloat16),           # a second, nearly empty token tile
    (100, 192, 608, 96, 640, torch.float16),        # narrow first rank, two slabs (wide + narrow) of the second
    (70, 128, 528, 784, 128, torch.bfloat16),       # the other way round; F ends inside a 512-wide chunk
    (257, 320, 1040, 272, 1024, torch.float16),     # odd number of 16-row steps in a narrow block, maximum second rank
])
def test_ffn_as_one_kernel_edge_shapes(fb, T, D, F, r1, r2, dt):
    """Shapes chosen around the kernel's block boundaries (32-token tiles, 256- and 512-column blocks, 16- and 32-row
    steps), with different ranks for the two factors: every element against the oracle."""
    g = torch.Generator().manual_seed(T * 1000 + r1 + r2)
    rn = lambda *shape, scale=1.0: (torch.randn(*shape, generator=g) * scale).to(dt)
    X = rn(1, T, D)
    raw = {"w1": (rn(D, r1, scale=D ** -0.5), rn(r1, F, scale=r1 ** -0.5), rn(F, scale=0.02)),
           "w2": (rn(F, r2, scale=F ** -0.5), rn(r2, D, scale=r2 ** -0.5), rn(D, scale=0.02))}
    fac = {k: fb.Factor(*(t.to(DEV) for t in v)).with_tiled(True, True) for k, v in raw.items()}
    ora = {k: dict(U=v[0].double().numpy(), V=v[1].double().numpy(), b=v[2].double().numpy()) for k, v in raw.items()}
    d = fb.make_desc(1, T, D, D // 64, F, dt, torch.float32, norm="none")
    got = fb.fsvd_ffn_v2(d, X.to(DEV), fac["w1"], fac["w2"]).cpu().numpy()
    ref = O.ffn(X.double().numpy(), ora["w1"], ora["w2"])
    assert np.isfinite(got).all()
    assert rel_err(got, ref) < TOL["ffn"]


def test_ffn_as_one_kernel_activations_and_types(fb):
    """Other activation functions, 16-bit output and missing biases."""
    w, inp, dev = workload("tiny_pad", fb, "tiled")
    for act in ("gelu_tanh", "relu"):
        d = fb.make_desc(w.B, w.M, w.D, w.H, w.F, dev["X"].dtype, torch.float32, act=act)
        assert rel_err(fb.fsvd_ffn_v2(d, dev["X"], dev["w1"], dev["w2"]).cpu().numpy(),
                       O.ffn(inp["X"], inp["w1"], inp["w2"], act=act)) < TOL["ffn"]
    d16 = fb.make_desc(w.B, w.M, w.D, w.H, w.F, dev["X"].dtype, torch.float16)
    ref = oracle_call(inp, "ffn")
    got16 = fb.fsvd_ffn_v2(d16, dev["X"], dev["w1"], dev["w2"])
    assert got16.dtype == torch.float16 and rel_err(got16.float().cpu().numpy(), ref) < TOL["ffn"] + 1e-3
    w1, w2 = dev["w1"], dev["w2"]
    nobias = [fb.Factor(f.U, f.V, None, f.U_tiled, f.V_tiled) for f in (w1, w2)]
    zero = [dict(inp[k], b=np.zeros_like(inp[k]["b"])) for k in ("w1", "w2")]
    assert rel_err(fb.fsvd_ffn_v2(dev["desc"], dev["X"], *nobias).cpu().numpy(), O.ffn(inp["X"], *zero)) < TOL["ffn"]


@pytest.mark.parametrize("name", ["cfg1_bert_base_b2_m128", "cfg2u_bert_base_b16_m512_pad_unit", "cfg3_bert_large_b32_m512_r128",
                                  "cfg3_bert_large_b32_m512_r512", "cfg4_long_b4_m8192", "ffn_grid_b16_m512_r384",
                                  "v2_llm_width_r1024"])
def test_ffn_as_one_kernel_full_size_sampled(fb, name):
    """The one-kernel FFN at benchmark sizes (32- and 64-token variants), sampled rows against the oracle."""
    w, inp, dev = workload(name, fb, "tiled")
    got = gpu_call(dev, "ffn_v2").cpu().numpy()
    assert np.isfinite(got).all()
    for b in (0, w.B - 1):
        rows = sample_rows(w, 10, seed=b)
        assert rel_err(got[b, rows], oracle_rows(inp, b, rows, "ffn")) < tol_for(w, "ffn"), (name, b)


def test_full_size_padding_property(fb):
    """Tokens at masked key positions cannot influence the context of any row (bitwise)."""
    w, inp, dev = workload("cfg2u_bert_base_b16_m512_pad_unit", fb)
    a = gpu_call(dev, "attention")
    X2 = dev["X"].clone()
    kl = inp["key_len"]
    for b in range(w.B):
        X2[b, kl[b]:] = torch.randn_like(X2[b, kl[b]:])
    dev2 = dict(dev, X=X2)
    a2 = gpu_call(dev2, "attention")
    for b in range(w.B):
        assert torch.equal(a[b, :kl[b]], a2[b, :kl[b]])


def test_full_size_causal_prefix_property(fb):
    """Under the causal mask, outputs at positions < p do not depend on tokens >= p (bitwise)."""
    w, inp, dev = workload("cfg5_llm_b1_m4096_causal", fb)
    a = gpu_call(dev, "layer")
    p = 1500
    X2 = dev["X"].clone()
    X2[:, p:] = torch.randn_like(X2[:, p:])
    a2 = gpu_call(dict(dev, X=X2), "layer")
    assert torch.equal(a[:, :p], a2[:, :p])
    assert not torch.equal(a[:, p:], a2[:, p:])


# ------------------------------------------------------------------ edge cases
def _run_custom(fb, w, mutate=None, **desc_kw):
    inp = W.make_inputs(w)
    if mutate:
        mutate(inp)
    dev = fb.to_device(inp, DEV)
    if desc_kw:
        base = dict(B=w.B, M=w.M, D=w.D, H=w.H, F=w.F, io_dtype=dev["X"].dtype, causal=inp["causal"],
                    key_len=dev["key_len"], norm=w.norm, ln_eps=w.ln_eps)
        base.update(desc_kw)
        dev["desc"] = fb.make_desc(**base)
    return inp, dev


def test_single_token_sequences(fb):
    w = W.get_workload("tiny_h2_d64", B=3, M=1)
    inp, dev = _run_custom(fb, w)
    for part in ("attention", "ffn", "layer"):
        assert rel_err(gpu_call(dev, part).cpu().numpy(), oracle_call(inp, part)) < tol_for(w, part) * 2


@pytest.mark.parametrize("name", ["ph_tiny_r16", "ph_tiny_d128_r64"])
def test_per_head_factors_edge_sequences(fb, name):
    """The absorbed schedule on single-token sequences, on lengths that end one key into a tile or a step, with one
    visible key, and with a causal mask on top of the padding."""
    for M in (1, 33, 129):
        w = W.get_workload(name, B=3, M=M, min_len=1)
        inp, dev = _run_custom(fb, w)
        for part in ("attention", "layer"):
            ref = oracle_call(inp, part)
            tol = attn_block_tol(w, ref) if part == "attention" else TOL_LAYER
            assert rel_err(gpu_call(dev, part).cpu().numpy(), ref) < tol * (2 if M == 1 else 1)
    w = W.get_workload(name, B=3, M=300, min_len=1)
    def mut(inp):
        inp["key_len"][:] = [1, 300, 129]
        inp["causal"] = True
    inp, dev = _run_custom(fb, w, mut)
    got = gpu_call(dev, "attention").cpu().numpy()
    ref = oracle_call(inp, "attention")
    assert np.isfinite(got).all()
    assert rel_err(got, ref) < max(attn_block_tol(w, ref), TOL["attention_causal"])


def test_key_len_one_and_full(fb):
    w = W.get_workload("tiny_pad")
    def mut(inp):
        inp["key_len"][:] = [1, w.M, 97]
    inp, dev = _run_custom(fb, w, mut)
    got = gpu_call(dev, "attention").cpu().numpy()
    ref = oracle_call(inp, "attention")
    assert rel_err(got, ref) < TOL["attention"]
    # with a single visible key every context row is that key's value vector
    v0 = O.factored_linear(O.factored_linear(inp["X"][0, 0], inp["v"]), inp["o"])
    assert np.abs(got[0] - v0[None, :]).max() < 5e-3 * np.abs(v0).max()


def test_causal_and_padding_combined(fb):
    w = W.get_workload("small_multi_qblock", mask="padding")
    inp = W.make_inputs(w)
    inp["causal"] = True
    dev = fb.to_device(inp, DEV)
    got = gpu_call(dev, "attention").cpu().numpy()
    assert rel_err(got, oracle_call(inp, "attention")) < TOL["attention_causal"]


def test_ragged_lengths_and_minimum_rank(fb):
    for M, r in ((33, 16), (129, 16), (257, 32)):
        w = W.get_workload("tiny_h2_d64", M=M, r_attn=r, r_ffn=16, B=1)
        inp, dev = _run_custom(fb, w)
        assert rel_err(gpu_call(dev, "layer").cpu().numpy(), oracle_call(inp, "layer")) < TOL_LAYER


def test_no_bias_custom_scale_and_activations(fb):
    w = W.get_workload("tiny_h2_d64")
    inp = W.make_inputs(w)
    dev = fb.to_device(inp, DEV)
    for n in ("q", "k", "v", "o", "w1", "w2"):
        inp[n]["b"] = None
        dev[n].b = None
    for act in ("gelu_tanh", "relu"):
        d = fb.make_desc(w.B, w.M, w.D, w.H, w.F, dev["X"].dtype, softmax_scale=0.05, act=act, norm=w.norm)
        dev["desc"] = d
        got = gpu_call(dev, "layer").cpu().numpy()
        a = (inp["q"], inp["k"], inp["v"], inp["o"])
        ref = O.layer(inp["X"], *a, (inp["ln1_gamma"], inp["ln1_beta"]), inp["w1"], inp["w2"],
                      (inp["ln2_gamma"], inp["ln2_beta"]), w.H, norm=w.norm, scale=0.05, act=act, eps=w.ln_eps)
        assert rel_err(got, ref) < TOL_LAYER


@pytest.mark.parametrize("name", ["ph_tiny_r16", "ph_tiny_d128_r48_causal"])
def test_per_head_factors_without_biases_and_with_a_caller_scale(fb, name):
    """The absorbed schedule folds b_q into the absorbed queries and adds b_v at the end: absent biases must read as
    zeros there too, and a caller's softmax scale must reach the absorbed queries."""
    w = W.get_workload(name)
    inp = W.make_inputs(w)
    dev = fb.to_device(inp, DEV)
    for n in ("q", "k", "v", "o"):
        inp[n]["b"] = None
        dev[n].b = None
    dev["desc"] = fb.make_desc(w.B, w.M, w.D, w.H, w.F, dev["X"].dtype, softmax_scale=0.07, key_len=dev["key_len"],
                               causal=(w.mask == "causal"), norm=w.norm, ln_eps=w.ln_eps)
    got = gpu_call(dev, "attention").cpu().numpy()
    ref = O.attention_per_head(inp["X"], inp["q"], inp["k"], inp["v"], inp["o"], w.H, inp["causal"], inp["key_len"], 0.07)
    assert np.isfinite(got).all()
    assert rel_err(got, ref) < attn_block_tol(w, ref)


@pytest.mark.parametrize("name,weights", [("cfg1_bert_base_b2_m128", "tiled"), ("tiny_causal_d128", "row"),
                                          ("ph_tiny_r48_causal", "row")])
def test_layer_replays_from_a_hip_graph(fb, name, weights):
    """The library only enqueues kernels on the caller's stream (no allocation, no memset, no host synchronisation), so
    a layer call with a caller workspace can be captured into a HIP graph: every replay on new inputs in the same
    buffers must equal the eager call on those inputs, with eager work and synchronisations between the replays."""
    w, inp, dev = workload(name, fb, weights)
    per_head = isinstance(dev["q"], fb.HeadFactor)
    layer = fb.fsvd_layer_heads if per_head else fb.fsvd_layer
    size = fb.fsvd_layer_heads_workspace if per_head else fb.fsvd_layer_workspace
    ranks = [dev[n].rank for n in ("q", "k", "v", "o", "w1", "w2")]
    ws = torch.empty(size(dev["desc"], *ranks), dtype=torch.uint8, device=DEV)
    x = dev["X"].clone()
    out = torch.empty(x.shape, dtype=torch.float32, device=DEV)
    args = (dev["q"], dev["k"], dev["v"], dev["o"], dev["ln1_gamma"], dev["ln1_beta"], dev["w1"], dev["w2"],
            dev["ln2_gamma"], dev["ln2_beta"])
    layer(dev["desc"], x, *args, out=out, workspace=ws)            # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        layer(dev["desc"], x, *args, out=out, workspace=ws)
    gen = torch.Generator(device=DEV).manual_seed(11)
    for k in range(3):
        x.copy_(torch.randn(x.shape, generator=gen, device=DEV).to(x.dtype))
        want = layer(dev["desc"], x, *args)
        torch.cuda.synchronize()
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want), k


@pytest.mark.parametrize("odt,eps", [(torch.float16, 2.0 ** -11), (torch.bfloat16, 2.0 ** -8)])
def test_sixteen_bit_outputs_round_the_fp32_result(fb, odt, eps):
    w, inp, dev = workload("tiny_pad", fb)
    ref32 = gpu_call(dev, "layer")
    d = dev["desc"]
    d16 = fb.make_desc(w.B, w.M, w.D, w.H, w.F, dev["X"].dtype, out_dtype=odt, key_len=dev["key_len"], norm=w.norm,
                       ln_eps=w.ln_eps)
    got = gpu_call(dict(dev, desc=d16), "layer")
    assert got.dtype == odt
    assert torch.equal(got, ref32.to(odt))


@pytest.mark.parametrize("odt", [torch.float16, torch.bfloat16])
@pytest.mark.parametrize("name", ["fuse_d768", "fuse_d256_causal"])
def test_sixteen_bit_outputs_of_the_fused_projection_and_layernorm(fb, name, odt):
    """The one-kernel hand-off (prepacked weights, at least 256 tokens) writes the layer's 16-bit output itself: the
    fp32 result of the same path, rounded to nearest."""
    w, inp, dev = workload(name, fb, "tiled")
    ref32 = gpu_call(dev, "layer")
    d16 = fb.make_desc(w.B, w.M, w.D, w.H, w.F, dev["X"].dtype, out_dtype=odt, key_len=dev["key_len"], norm=w.norm,
                       ln_eps=w.ln_eps, causal=(w.mask == "causal"))
    got = gpu_call(dict(dev, desc=d16), "layer")
    assert got.dtype == odt
    assert torch.equal(got, ref32.to(odt))


def test_run_to_run_determinism(fb):
    """No atomics anywhere: two runs are bitwise equal."""
    w, inp, dev = workload("small_multi_qblock", fb)
    for part in ("attention", "ffn", "layer"):
        assert torch.equal(gpu_call(dev, part), gpu_call(dev, part))


def test_layer_and_one_kernel_ffn_replay_from_a_captured_graph(fb):
    """The library only launches kernels on the caller's stream (no allocation, no memset, no host synchronisation), so a
    caller may capture a call in a graph: replays with new input values, with eager work in between, equal the eager
    results bit for bit."""
    w, inp, dev = workload("tiny_pad", fb, "tiled")
    d = dev["desc"]
    args = (dev["q"], dev["k"], dev["v"], dev["o"], dev["ln1_gamma"], dev["ln1_beta"], dev["w1"], dev["w2"],
            dev["ln2_gamma"], dev["ln2_beta"])
    need = fb.fsvd_layer_workspace(d, w.r_attn, w.r_attn, w.r_attn, w.r_attn, w.r_ffn, w.r_ffn)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    X = dev["X"].clone()
    out = torch.empty((w.B, w.M, w.D), dtype=torch.float32, device=DEV)
    out2 = torch.empty_like(out)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up outside the capture, as torch asks
        fb.fsvd_layer(d, X, *args, out=out, workspace=ws)
        fb.fsvd_ffn_v2(d, X, dev["w1"], dev["w2"], out=out2)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fb.fsvd_layer(d, X, *args, out=out, workspace=ws)
        fb.fsvd_ffn_v2(d, X, dev["w1"], dev["w2"], out=out2)
    gen = torch.Generator(device=DEV).manual_seed(7)
    for rep in range(3):
        X.copy_(torch.randn(X.shape, generator=gen, device=DEV).to(X.dtype))
        graph.replay()
        torch.cuda.synchronize()
        got, got2 = out.clone(), out2.clone()
        eager = fb.fsvd_layer(d, X, *args)             # eager work between the replays (own workspace and output)
        eager2 = fb.fsvd_ffn_v2(d, X, dev["w1"], dev["w2"])
        torch.cuda.synchronize()
        assert torch.equal(got, eager), rep
        assert torch.equal(got2, eager2), rep


def test_rank_padding_invariance(fb):
    """Zero-padding every rank to a larger multiple of 16 leaves the result bitwise unchanged."""
    w = W.get_workload("tiny_h2_d64")
    inp = W.make_inputs(w)
    dev = fb.to_device(inp, DEV)
    base = gpu_call(dev, "layer")
    pad = 32
    for n in ("q", "k", "v", "o", "w1", "w2"):
        f = dev[n]
        f.U = torch.nn.functional.pad(f.U, (0, pad)).contiguous()
        f.V = torch.nn.functional.pad(f.V, (0, 0, 0, pad)).contiguous()
    assert torch.equal(gpu_call(dev, "layer"), base)


# ------------------------------------------------------------------ range precondition of bf16 storage, measured memory
def _f16_toward_zero(x32):
    """fp32 -> fp16 with rounding toward zero and saturation at +-65504 (the documented conversion of bf16 factors)."""
    x32 = np.asarray(x32, dtype=np.float32)
    with np.errstate(over="ignore"):
        h = x32.astype(np.float16)
    h = np.where(np.isinf(h), np.float16(65504.0) * np.sign(x32).astype(np.float16), h)
    away = np.abs(h.astype(np.float32)) > np.abs(x32)
    return np.where(away, np.nextafter(h, np.float16(0.0)), h).astype(np.float16)


@pytest.mark.parametrize("tiled", [False, True])
def test_bf16_factor_values_outside_the_fp16_range_saturate_or_truncate(fb, tiled):
    """A bf16 factor element beyond fp16's range (1e5, -3e38) saturates to +-65504 and one below its normal range (1e-6,
    3e-8, 1e-9) is truncated toward zero on fp16's subnormal grid; the expectation is the oracle's projection of the
    weights converted that way on the CPU.  Nothing is flagged: the range is the caller's precondition."""
    K, N, T = 64, 48, 40
    rng = np.random.default_rng(11)
    Wm = (rng.standard_normal((K, N)) / 8).astype(np.float32)
    odd = [1.0e5, -3.0e38, 65504.0, 7.0e4, 1.0e-6, -1.0e-6, 3.0e-8, 1.0e-9, -2.0 ** -14, 6.1e-5]
    for i, v in enumerate(odd):
        Wm[3 + 5 * i, (7 * i) % N] = v
    Wb = torch.from_numpy(Wm).to(torch.bfloat16)
    W16 = _f16_toward_zero(Wb.float().numpy())
    assert np.isfinite(W16).all() and np.abs(W16).max() == 65504.0 and (W16 == 0).sum() >= 1
    A = torch.from_numpy((rng.standard_normal((T, K)) / 4).astype(np.float32)).to(torch.float16)
    ref = O.rank_projection(A.double().numpy(), W16.astype(np.float64))
    Wd = Wb.to(DEV)
    got = (fb.fsvd_linear_tiled(A.to(DEV), fb.fsvd_pack_tiled(Wd), N, out_dtype=torch.float32) if tiled
           else fb.fsvd_linear(A.to(DEV), Wd, out_dtype=torch.float32)).cpu().numpy()
    assert np.isfinite(got).all()
    # element-wise: fp32 accumulation of exactly representable products, sums up to ~1e5 in magnitude
    assert np.abs(got - ref).max() <= 2e-6 * np.abs(ref).max()
    if tiled:      # the prepacked image holds exactly those fp16 values
        img = fb.fsvd_pack_tiled(Wd).view(torch.float16).cpu().numpy()
        assert np.array_equal(img.view(np.uint16), expected_tile_images(W16).view(np.uint16))


def test_bf16_activation_values_outside_the_fp16_range_saturate_or_truncate(fb):
    """The same conversion applies to a bf16 activation, whether a projection reads it row-major or a layer packs it
    into the fragment-major layout first: 1e5 is used as 65504, 1e-6 as the fp16 subnormal below it."""
    T, K, N = 70, 64, 32
    rng = np.random.default_rng(12)
    A = (rng.standard_normal((T, K)) / 4).astype(np.float32)
    A[5, 3], A[69, 63], A[33, 40], A[34, 41], A[0, 0] = 1.0e5, -1.0e5, 1.0e-6, -3.0e-8, 1.0e-9
    Ab = torch.from_numpy(A).to(torch.bfloat16)
    A16 = _f16_toward_zero(Ab.float().numpy())
    Wm = torch.from_numpy((rng.standard_normal((K, N)) / 8).astype(np.float32)).to(torch.bfloat16)
    ref = O.rank_projection(A16.astype(np.float64), Wm.double().numpy())
    got = fb.fsvd_linear(Ab.to(DEV), Wm.to(DEV), out_dtype=torch.float32).cpu().numpy()
    assert np.isfinite(got).all()
    assert np.abs(got - ref).max() <= 2e-6 * np.abs(ref).max()
    back = fb.fsvd_unpack_fm(fb.fsvd_pack_fm(Ab.to(DEV)), T, K, torch.float32).cpu().numpy()
    assert np.array_equal(back, A16.astype(np.float32))


def test_workspace_is_the_whole_transient_footprint(fb):
    """The library takes no device memory of its own: with workspace and output allocated by the caller's allocator
    inside the measured region, the allocator's peak is workspace + output (to its 512-byte rounding), and a call on
    preallocated buffers leaves the device's free memory unchanged."""
    name = "cfg1_bert_base_b2_m128"
    w, inp, dev = workload(name, fb, "tiled")
    d = dev["desc"]
    args = (dev["X"], dev["q"], dev["k"], dev["v"], dev["o"], dev["ln1_gamma"], dev["ln1_beta"], dev["w1"], dev["w2"],
            dev["ln2_gamma"], dev["ln2_beta"])
    need = fb.fsvd_layer_workspace(d, w.r_attn, w.r_attn, w.r_attn, w.r_attn, w.r_ffn, w.r_ffn)
    out_bytes = w.T * w.D * 4
    fb.fsvd_layer(d, *args)                       # warm-up: loads the kernels' code objects
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    torch.cuda.reset_peak_memory_stats()
    base = torch.cuda.memory_allocated()
    out = fb.fsvd_layer(d, *args)                 # the binding allocates `out` and the workspace with torch
    torch.cuda.synchronize()
    peak = torch.cuda.max_memory_allocated() - base
    _report(f"MEMORY {name}: workspace {need} B + output {out_bytes} B = {need + out_bytes}; allocator peak {peak} B")
    assert need + out_bytes <= peak <= need + out_bytes + 2 * 512
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    fb.fsvd_layer(d, *args, out=out, workspace=ws)
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free1 == free0
    # and the workspace is strictly below the unfused dataflow's transient buffers (fp32 stream, context, Q/K/V or hidden)
    T, D, F, ra, rf = w.T, w.D, w.F, w.r_attn, w.r_ffn
    unfused = T * D * 4 + T * D * 2 + max(3 * T * ra * 2 + 3 * T * D * 2, 2 * T * rf * 2 + T * F * 2)
    assert need < unfused
