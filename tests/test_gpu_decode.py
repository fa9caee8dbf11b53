"""GPU parity of the decoding step against a rank-space KV cache: the library through its C ABI against the oracle's
plain definition (full-width keys and values rebuilt from the cache, nothing absorbed), plus the cache's byte layout."""
import numpy as np
import pytest
import torch

from oracle import fsvd_oracle as O
from paper_2508_01506_amd import workloads as W
from fsvd_testing import rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
# The step hands fp16 tensors from stage to stage like the prefill attention block (rank projections, the absorbed
# queries, the probabilities, the per-part sums, the context): same derived bound as for that block.
TOL_DECODE = 6e-3


def assert_step_close(got, ref, what=""):
    """Every sequence is a problem of its own (its context length sets the scale of its output: attention over many
    keys averages the values down), so the gate is applied per sequence: max |err| / RMS(ref) of that sequence below the
    derived bound, or, for outputs of small scale, the same absolute fp16 hand-off noise (1e-3) relative to that RMS."""
    for b in range(ref.shape[0]):
        rms = float(np.sqrt(np.mean(np.asarray(ref[b], dtype=np.float64) ** 2)))
        err = rel_err(got[b], ref[b])
        assert err < max(TOL_DECODE, 1.0e-3 / rms), (what, b, err, rms)


@pytest.fixture(scope="module")
def fb():
    from paper_2508_01506_amd import binding
    binding.lib()
    assert torch.cuda.is_available(), "these tests need the GPU"
    return binding


def device_inputs(fb, inp):
    w = inp["workload"]
    dt = torch.float16 if w.dtype == "fp16" else torch.bfloat16
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(device=DEV, dtype=dt).contiguous()
    dev = {n: fb.Factor(up(inp[n]["U"]), up(inp[n]["V"]), up(inp[n]["b"])) for n in "qkvo"}
    dev["x_new"] = up(inp["x_new"])
    dev["desc"] = fb.make_desc(w.B, w.t_max, w.D, w.H, 16, dt, torch.float32)
    kc, vc = fb.fsvd_decode_new_caches(w.B, w.t_max, w.r, w.r, DEV)
    zero = torch.zeros(w.B, dtype=torch.int32, device=DEV)
    # the whole history is loaded, rows past each sequence's length included: they must be ignored (and the row at
    # position lens[b] is overwritten by the step)
    fb.fsvd_decode_cache_write(kc, 0, w.t_max, torch.from_numpy(inp["Pk"]).to(DEV, torch.float16), zero)
    fb.fsvd_decode_cache_write(vc, 1, w.t_max, torch.from_numpy(inp["Pv"]).to(DEV, torch.float16), zero)
    dev["kc"], dev["vc"] = kc, vc
    dev["lens"] = torch.from_numpy(inp["lens"]).to(DEV)
    return dev


def k_cache_image(P, t_max):
    """Fragment-major image of P [t, r] padded to t_max tokens (the documented K-cache layout of one sequence)."""
    t, r = P.shape
    tiles, kch = (t_max + 31) // 32, (r + 63) // 64
    img = np.zeros((tiles, kch, 4, 64, 8), np.float16)
    for tok in range(t):
        for rho in range(0, r, 8):
            off = rho % 64
            img[tok // 32, rho // 64, (off // 8) % 4, 32 * (off // 32) + tok % 32] = P[tok, rho:rho + 8]
    return img.reshape(-1)


def v_cache_image(P, t_max):
    """The documented V-cache layout of one sequence: key tile x rank tile blocks of 2 KiB in operand order."""
    t, r = P.shape
    ktiles = (t_max + 31) // 32
    img = np.zeros((ktiles, r // 32, 2, 64, 8), np.float16)
    slot_keys = [0, 1, 2, 3, 8, 9, 10, 11]
    for tok in range(t):
        kq = tok % 32
        s, o = kq // 16, kq % 16
        g = (o // 4) % 2
        i = slot_keys.index(o - 4 * g)
        for rho in range(r):
            img[tok // 32, rho // 32, s, 32 * g + rho % 32, i] = P[tok, rho]
    return img.reshape(-1)


def test_cache_write_produces_the_documented_layouts(fb):
    """Byte work, bit-exact: a bulk load and two ragged appends against images written from the layouts' definitions."""
    rng = np.random.default_rng(3)
    B, t_max, r = 2, 70, 64
    hist = rng.standard_normal((B, 40, r)).astype(np.float16)
    extra = rng.standard_normal((B, 3, r)).astype(np.float16)
    kc, vc = fb.fsvd_decode_new_caches(B, t_max, r, r, DEV)
    assert kc.numel() == B * 3 * 1 * 4096 and vc.numel() == B * 2 * 3 * 2048
    zero = torch.zeros(B, dtype=torch.int32, device=DEV)
    start = torch.tensor([40, 37], dtype=torch.int32, device=DEV)       # the second sequence overwrites 3 of its rows
    for cache, which in ((kc, 0), (vc, 1)):
        fb.fsvd_decode_cache_write(cache, which, t_max, torch.from_numpy(hist).to(DEV), zero)
        fb.fsvd_decode_cache_write(cache, which, t_max, torch.from_numpy(extra).to(DEV), start)
    want = [np.concatenate([hist[0], extra[0]]), np.concatenate([hist[1][:37], extra[1]])]
    got_k = kc.view(torch.float16).cpu().numpy().reshape(B, -1)
    got_v = vc.view(torch.float16).cpu().numpy().reshape(B, -1)
    for b in range(B):
        assert np.array_equal(got_k[b].view(np.uint16), k_cache_image(want[b], t_max).view(np.uint16))
        assert np.array_equal(got_v[b].view(np.uint16), v_cache_image(want[b], t_max).view(np.uint16))
    # rows that would fall past the capacity are dropped, nothing else is touched
    before = kc.clone()
    fb.fsvd_decode_cache_write(kc, 0, t_max, torch.from_numpy(extra).to(DEV), torch.tensor([t_max, t_max + 5], dtype=torch.int32, device=DEV))
    assert torch.equal(kc, before)


def run_step(fb, dev):
    return fb.fsvd_decode_attention(dev["desc"], dev["x_new"], dev["q"], dev["k"], dev["v"], dev["o"], dev["kc"], dev["vc"],
                                    dev["lens"]).cpu().numpy()


@pytest.mark.parametrize("name", ["decode_tiny_d64", "decode_tiny_d128", "decode_tiny_b70", "decode_base_b32_t1024_r256"])
def test_decode_step_every_element(fb, name):
    """Ragged cache lengths from an empty cache to a full one; every output element against the oracle."""
    inp = W.make_decode_inputs(W.DECODE_WORKLOADS[name])
    w = inp["workload"]
    dev = device_inputs(fb, inp)
    got = run_step(fb, dev)
    ref, pk_new, pv_new = O.decode_attention(inp["x_new"], inp["Pk"], inp["Pv"], inp["lens"], inp["q"], inp["k"], inp["v"], inp["o"], w.H)
    assert np.isfinite(got).all()
    assert_step_close(got, ref, name)
    # the step appended the new token's rows: a second step on the advanced lengths sees them
    nxt = np.minimum(inp["lens"] + 1, w.t_max - 1).astype(np.int32)
    Pk2, Pv2 = inp["Pk"].copy(), inp["Pv"].copy()
    for b in range(w.B):
        Pk2[b, inp["lens"][b]] = pk_new[b].astype(np.float16)
        Pv2[b, inp["lens"][b]] = pv_new[b].astype(np.float16)
    dev["lens"] = torch.from_numpy(nxt).to(DEV)
    got2 = run_step(fb, dev)
    ref2, _, _ = O.decode_attention(inp["x_new"], Pk2, Pv2, nxt, inp["q"], inp["k"], inp["v"], inp["o"], w.H)
    assert_step_close(got2, ref2, name + " second step")


@pytest.mark.parametrize("name", ["decode_llm_b16_t4096_r1024", "decode_llm_b64_t2048_r512"])
def test_decode_step_benchmark_sizes_sampled_sequences(fb, name):
    """At the sizes bench.py times, in its launch configuration: whole output rows of sampled sequences."""
    inp = W.make_decode_inputs(W.DECODE_WORKLOADS[name])
    w = inp["workload"]
    dev = device_inputs(fb, inp)
    got = run_step(fb, dev)
    assert np.isfinite(got).all()
    for b in (0, w.B // 2, w.B - 1):
        sl = slice(b, b + 1)
        ref, _, _ = O.decode_attention(inp["x_new"][sl], inp["Pk"][sl], inp["Pv"][sl], inp["lens"][sl], inp["q"], inp["k"],
                                       inp["v"], inp["o"], w.H)
        assert_step_close(got[sl], ref, name)


def test_decode_core_rank_space_context(fb):
    """The pass over the cache alone: u = softmax(P_k W^T) P_v per head, with the absorbed queries given."""
    rng = np.random.default_rng(11)
    B, t_max, H, D, r_k, r_v = 4, 900, 12, 768, 192, 160
    lens = np.array([1, 33, 512, 900], np.int32)
    Pk = rng.standard_normal((B, t_max, r_k)).astype(np.float16)
    Pv = rng.standard_normal((B, t_max, r_v)).astype(np.float16)
    Wq = (rng.standard_normal((B, H, r_k)) * 0.15).astype(np.float16)     # log2-domain scores of a few units
    kc, vc = fb.fsvd_decode_new_caches(B, t_max, r_k, r_v, DEV)
    zero = torch.zeros(B, dtype=torch.int32, device=DEV)
    fb.fsvd_decode_cache_write(kc, 0, t_max, torch.from_numpy(Pk).to(DEV), zero)
    fb.fsvd_decode_cache_write(vc, 1, t_max, torch.from_numpy(Pv).to(DEV), zero)
    Wpad = np.zeros((B, 32, r_k), np.float16)
    Wpad[:, :H] = Wq
    Wfm = torch.cat([fb.fsvd_pack_fm(torch.from_numpy(Wpad[b]).to(DEV)) for b in range(B)])
    d = fb.make_desc(B, t_max, D, H, 16, torch.float16)
    got = fb.fsvd_decode_attention_core(d, r_k, r_v, Wfm, kc, vc, torch.from_numpy(lens).to(DEV)).cpu().numpy()
    for b in range(B):
        n = lens[b]
        s = Pk[b, :n].astype(np.float64) @ Wq[b].astype(np.float64).T * np.log(2.0)   # W carries log2(e): undo it for exp
        a = O.softmax_rows(s.T)
        ref = a @ Pv[b, :n].astype(np.float64)
        assert rel_err(got[b], ref) < 3e-3, b


@pytest.mark.parametrize("case", ["one_long_rest_empty", "all_equal", "single_sequence", "sixty_four_ragged", "more_than_sixty_four",
                                  "all_empty_but_last"])
def test_decode_core_balanced_split_over_ragged_batches(fb, case):
    """The pass over the cache deals its workgroups to the sequences in proportion to their key tiles (and falls back to
    equal parts above 64 sequences): batches whose lengths are as uneven as they can be, against the plain softmax."""
    rng = np.random.default_rng(sum(map(ord, case)))
    H, D, r_k, r_v, t_max = 8, 512, 128, 96, 700
    lens = {
        "one_long_rest_empty": [700] + [0] * 15,
        "all_equal": [333] * 8,
        "single_sequence": [640],
        "sixty_four_ragged": [int(x) for x in np.random.default_rng(5).integers(0, 701, size=64)],
        "more_than_sixty_four": [int(x) for x in np.random.default_rng(6).integers(0, 701, size=80)],
        "all_empty_but_last": [0] * 31 + [97],
    }[case]
    B = len(lens)
    lens = np.array(lens, np.int32)
    Pk = rng.standard_normal((B, t_max, r_k)).astype(np.float16)
    Pv = rng.standard_normal((B, t_max, r_v)).astype(np.float16)
    Wq = (rng.standard_normal((B, H, r_k)) * 0.15).astype(np.float16)
    kc, vc = fb.fsvd_decode_new_caches(B, t_max, r_k, r_v, DEV)
    zero = torch.zeros(B, dtype=torch.int32, device=DEV)
    fb.fsvd_decode_cache_write(kc, 0, t_max, torch.from_numpy(Pk).to(DEV), zero)
    fb.fsvd_decode_cache_write(vc, 1, t_max, torch.from_numpy(Pv).to(DEV), zero)
    Wpad = np.zeros((B, 32, r_k), np.float16)
    Wpad[:, :H] = Wq
    Wfm = torch.cat([fb.fsvd_pack_fm(torch.from_numpy(Wpad[b]).to(DEV)) for b in range(B)])
    d = fb.make_desc(B, t_max, D, H, 16, torch.float16)
    got = fb.fsvd_decode_attention_core(d, r_k, r_v, Wfm, kc, vc, torch.from_numpy(lens).to(DEV)).cpu().numpy()
    assert np.isfinite(got).all()
    for b in range(B):
        n = int(lens[b])
        if n == 0:
            assert not got[b].any(), b            # no keys: the context is zero
            continue
        s = Pk[b, :n].astype(np.float64) @ Wq[b].astype(np.float64).T * np.log(2.0)
        ref = O.softmax_rows(s.T) @ Pv[b, :n].astype(np.float64)
        assert rel_err(got[b], ref) < 6e-3, (case, b, n)      # the attention-block bound: probabilities and u are fp16 hand-offs
