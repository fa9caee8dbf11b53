"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, validates arguments before touching a device, and sizes workspaces as documented."""
import ctypes as C
import os
import re

import numpy as np

import pytest
import torch

from paper_2508_01506_amd import binding as fb
from paper_2508_01506_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, INVALID, UNSUPPORTED, WORKSPACE, DEVICE = range(5)


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "fsvd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fsvd_[a-z_0-9]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    L = fb.lib()
    names = declared_symbols()
    assert len(names) >= 14
    for n in names:
        assert hasattr(L, n), f"{n} declared in fsvd.h but not exported"
    assert sorted(fb.EXPORTS) == names
    assert L.fsvd_version() >= 100
    for code, frag in [(0, b"ok"), (1, b"invalid"), (2, b"unsupported"), (3, b"workspace"), (4, b"device")]:
        assert frag in L.fsvd_status_string(code)


def desc(**kw):
    base = dict(B=2, M=128, D=768, H=12, F=3072, io_dtype=torch.float16)
    base.update(kw)
    return fb.make_desc(**base)


def test_workspace_sizes_follow_the_documented_plan():
    up = lambda n: (n + 255) // 256 * 256
    fm = lambda T, K: ((T + 31) // 32) * ((K + 63) // 64) * 4096      # fragment-major fp16 [T, K]
    for w in W.WORKLOADS.values():
        d = fb.make_desc(w.B, w.M, w.D, w.H, w.F, torch.float16, norm=w.norm)
        T, D, ra, rf = w.T, w.D, w.r_attn, w.r_ffn
        assert fb.fsvd_fm_bytes(T, ra) == fm(T, ra)
        attn_rank = max(3 * up(fm(T, ra)), up(fm(T, ra)))                # P_q | P_k | P_v, later T_o in the same bytes
        attn = up(fm(T, D)) + attn_rank                                  # context (first the packed X) + rank scratch
        part = fb.fsvd_ffn_core_workspace(d, rf, rf)                     # fp32 partial sums of Z when the core splits F
        assert part % 256 == 0 and part <= up(T * w.F)                   # never more than half the hidden activation
        zpad = (rf + 63) // 64 * 64
        assert part == 0 or part % up(zpad * T * 4) == 0 or part == up(part)   # a whole number of [r2, T] fp32 slabs
        ffn = 2 * up(fm(T, rf)) + part                                   # P1 + Z (+ partial sums)
        assert fb.fsvd_attention_workspace(d, ra, ra, ra, ra) == attn
        assert fb.fsvd_ffn_workspace(d, rf, rf) == ffn
        stream = 0 if w.norm == "none" else up(T * D * 4)                # fp32 residual stream
        layer = stream + up(fm(T, D)) + max(attn_rank, ffn)
        assert fb.fsvd_layer_workspace(d, ra, ra, ra, ra, rf, rf) == layer
        # strictly below the unfused factored layer's transient buffers (same fp16 storage, same reuse):
        # that path also materialises Q, K, V [T, D] next to P and the hidden [T, F] next to P1 and Z
        assert attn < attn + 3 * T * D * 2 and ffn < ffn + T * w.F * 2
        unfused = stream + T * D * 2 + max(3 * T * ra * 2 + 3 * T * D * 2, 2 * T * rf * 2 + T * w.F * 2)
        if T >= 256 and T % 32 == 0:     # padding of tiny shapes aside, the fused workspace is strictly smaller
            assert layer < unfused, (w.name, layer, unfused)


def test_workspace_query_rejects_bad_configurations():
    assert fb.fsvd_attention_workspace(desc(H=7), 64, 64, 64, 64) == 0          # D % H != 0
    assert fb.fsvd_attention_workspace(desc(D=96, H=3), 64, 64, 64, 64) == 0    # d_h = 32
    assert fb.fsvd_attention_workspace(desc(), 60, 64, 64, 64) == 0             # rank not a multiple of 16
    assert fb.fsvd_ffn_workspace(desc(F=0), 64, 64) == 0
    assert fb.fsvd_ffn_workspace(desc(B=0), 64, 64) == 0
    assert fb.fsvd_layer_workspace(desc(), 64, 64, 64, 64, 64, 0) == 0
    assert fb.fsvd_attention_workspace(desc(), 64, 64, 64, 64) > 0


def fac(i, r, o, U=256, V=256):
    return fb.fsvd_factor(U, V, 0, i, r, o)


def test_checks_report_the_documented_status_codes():
    L = fb.lib()
    d = desc()
    good = fac(768, 64, 768)
    chk = lambda dd, q, k, v, o: L.fsvd_attention_check(C.byref(dd), C.byref(q), C.byref(k), C.byref(v), C.byref(o))
    assert chk(d, good, good, good, good) == OK
    assert chk(d, fac(768, 64, 512), good, good, good) == INVALID        # wrong out_dim
    assert chk(d, good, fac(512, 64, 768), good, good) == INVALID        # wrong in_dim
    assert chk(d, good, good, fac(768, 0, 768), good) == INVALID         # rank 0
    assert chk(d, good, good, good, fac(768, 24, 768)) == UNSUPPORTED    # rank % 16
    assert chk(desc(D=96, H=3), fac(96, 16, 96), fac(96, 16, 96), fac(96, 16, 96), fac(96, 16, 96)) == UNSUPPORTED
    assert chk(desc(H=5), good, good, good, good) == INVALID
    assert chk(desc(B=-1), good, good, good, good) == INVALID
    bad_dtype = desc()
    bad_dtype.io_dtype = 2
    assert chk(bad_dtype, good, good, good, good) == INVALID
    big = desc(B=1 << 12, M=1 << 12)
    assert chk(big, good, good, good, good) == UNSUPPORTED
    w1, w2 = fac(768, 64, 3072), fac(3072, 64, 768)
    assert L.fsvd_ffn_check(C.byref(d), C.byref(w1), C.byref(w2)) == OK
    assert L.fsvd_ffn_check(C.byref(d), C.byref(w2), C.byref(w1)) == INVALID
    assert L.fsvd_ffn_check(C.byref(desc(F=3080)), C.byref(fac(768, 64, 3080)), C.byref(fac(3080, 64, 768))) == UNSUPPORTED


def test_compute_entry_points_validate_before_any_launch():
    """Null pointers, short or misaligned workspaces are rejected on the host (no GPU is needed to see it)."""
    L = fb.lib()
    d = desc()
    q = fac(768, 64, 768)
    need = fb.fsvd_attention_workspace(d, 64, 64, 64, 64)
    call = lambda X, out, ws, n: L.fsvd_attention(C.byref(d), X, C.byref(q), C.byref(q), C.byref(q), C.byref(q), out, ws, n, None)
    assert call(None, 256, 256, need) == INVALID
    assert call(256, None, 256, need) == INVALID
    assert call(256, 256, None, need) == WORKSPACE
    assert call(256, 256, 256, need - 1) == WORKSPACE
    assert call(256, 256, 257, need) == WORKSPACE               # not 256-byte aligned
    assert call(264, 256, 256, need) == INVALID                 # X not 16-byte aligned
    assert call(256, 260, 256, need) == INVALID                 # out not 16-byte aligned
    assert L.fsvd_attention(C.byref(d), 256, C.byref(fac(768, 64, 768, V=8)), C.byref(q), C.byref(q), C.byref(q), 256, 256, need, None) == INVALID
    nullU = fac(768, 64, 768, U=0)
    assert L.fsvd_attention(C.byref(d), 256, C.byref(nullU), C.byref(q), C.byref(q), C.byref(q), 256, 256, need, None) == INVALID
    w1, w2 = fac(768, 64, 3072), fac(3072, 64, 768)
    assert L.fsvd_ffn(C.byref(d), 256, C.byref(w1), C.byref(w2), 256, 256, 16, None) == WORKSPACE
    lneed = fb.fsvd_layer_workspace(d, 64, 64, 64, 64, 64, 64)
    layer = lambda g1: L.fsvd_layer(C.byref(d), 256, C.byref(q), C.byref(q), C.byref(q), C.byref(q), g1, 256,
                                    C.byref(w1), C.byref(w2), 256, 256, 256, 256, lneed, None)
    assert layer(None) == INVALID                               # LayerNorm parameters required unless norm == NONE
    assert L.fsvd_linear(16, 40, 16, 256, 0, 256, None, 0, None, 0, 256, 0, None) == UNSUPPORTED   # K % 16
    assert L.fsvd_linear(0, 32, 16, 256, 0, 256, None, 0, None, 0, 256, 0, None) == INVALID
    assert L.fsvd_layernorm(4, 16384, 256, 0, 256, 256, 0, 1e-5, 256, 2, None) == UNSUPPORTED
    assert L.fsvd_layernorm(4, 64, None, 0, 256, 256, 0, 1e-5, 256, 2, None) == INVALID
    # the FFN core splits D_ff for this small shape: it then needs its partial-sum workspace, and only then
    w1r, w2r = fac(768, 384, 3072), fac(3072, 384, 768)
    core_need = fb.fsvd_ffn_core_workspace(d, 384, 384)
    assert core_need > 0 and core_need % 256 == 0
    core = lambda ws, n: L.fsvd_ffn_core(C.byref(d), 256, C.byref(w1r), C.byref(w2r), 256, ws, n, None)
    assert core(None, 0) == WORKSPACE
    assert core(256, core_need - 256) == WORKSPACE
    assert L.fsvd_ffn_core(C.byref(d), None, C.byref(w1r), C.byref(w2r), 256, 256, core_need, None) == INVALID
    big = desc(B=32, M=512, D=1024, H=16, F=4096)                  # plenty of workgroups: no split, no workspace
    assert fb.fsvd_ffn_core_workspace(big, 256, 256) == 0


def test_tiled_weight_layout_contract():
    """Tile images: documented size, accepted only where the header says, both FFN streams alike, bad values rejected."""
    L = fb.lib()
    d = desc()
    assert fb.fsvd_tiled_bytes(128, 128) == 32768
    assert fb.fsvd_tiled_bytes(129, 136) == 4 * 32768
    assert fb.fsvd_tiled_bytes(2048, 16384) == 16 * 128 * 32768
    assert fb.fsvd_tiled_bytes(16, 12) == 0 and fb.fsvd_tiled_bytes(0, 16) == 0
    assert fb.fsvd_tiled_bytes(1 << 15, 1 << 15) == 0                     # would reach 2 GiB
    assert L.fsvd_pack_tiled(128, 128, None, 0, 256, None) == INVALID
    assert L.fsvd_pack_tiled(128, 128, 256, 2, 256, None) == INVALID     # fp32 weights are not a storage type
    assert L.fsvd_pack_tiled(128, 128, 264, 0, 256, None) == INVALID     # misaligned
    assert L.fsvd_pack_tiled(128, 12, 256, 0, 256, None) == UNSUPPORTED

    def lay(f, u=0, v=0):
        return fb.fsvd_factor(f.U, f.V, f.bias, f.in_dim, f.rank, f.out_dim, u, v)
    w1, w2 = fac(768, 64, 3072), fac(3072, 64, 768)
    ffn = lambda a, b: L.fsvd_ffn_check(C.byref(d), C.byref(a), C.byref(b))
    assert ffn(lay(w1, v=1), lay(w2, u=1)) == OK
    assert ffn(lay(w1, u=1, v=1), lay(w2, u=1, v=1)) == OK
    assert ffn(lay(w1, u=1), lay(w2, v=1)) == OK                          # the two plain projections, each on its own
    assert ffn(lay(w1, v=1), w2) == UNSUPPORTED                           # both streams of the fused core or neither
    assert ffn(w1, lay(w2, u=1)) == UNSUPPORTED
    assert ffn(lay(w1, v=2), lay(w2, u=2)) == INVALID                     # not a layout
    assert ffn(lay(w1, v=-1), w2) == INVALID
    q = fac(768, 64, 768)
    att = lambda a, b, c, o: L.fsvd_attention_check(C.byref(d), C.byref(a), C.byref(b), C.byref(c), C.byref(o))
    tv, tu = lay(q, v=1), lay(q, u=1)
    assert att(tv, tv, tv, q) == OK                                       # the rebuild weights V_q, V_k, V_v: all three
    assert att(tv, q, tv, q) == UNSUPPORTED                               # ... or none
    assert att(tu, tu, tu, lay(q, u=1, v=1)) == OK                        # likewise the three rank projections
    assert att(tu, tu, q, q) == UNSUPPORTED
    assert att(q, q, q, lay(q, v=1)) == OK                                # the output projection's factors are free
    heads = lambda a: L.fsvd_attention_heads(C.byref(d), 256, C.byref(a), C.byref(a), C.byref(a), C.byref(q), 256, 256, 1 << 40, None)
    assert heads(lay(fac(768, 32, 768), v=1)) == UNSUPPORTED              # V of per-head factors stays row-major
    assert L.fsvd_linear_tiled(16, 32, 16, 256, 0, 256, None, 0, None, 0, 264, 0, None) == INVALID   # C misaligned
    assert L.fsvd_linear_tiled(16, 40, 16, 256, 0, 256, None, 0, None, 0, 256, 0, None) == UNSUPPORTED


def test_ffn_with_static_scratch_contract():
    """fsvd_ffn_static validates like fsvd_ffn and refuses, before touching a device, a problem whose workspace would not
    fit the library's static scratch array."""
    L = fb.lib()
    d = desc()
    w1, w2 = fac(768, 64, 3072), fac(3072, 64, 768)
    call = lambda dd, a, b, x=256, out=256: L.fsvd_ffn_static(C.byref(dd), x, C.byref(a), C.byref(b), out, None)
    assert call(d, w1, w2, x=None) == INVALID
    assert call(d, w1, w2, out=264) == INVALID
    assert call(d, w2, w1) == INVALID
    assert call(d, fac(768, 24, 3072), w2) == UNSUPPORTED
    big = desc(B=1, M=4096, D=4096, H=32, F=16384)                         # the decoder shape: 192 MiB of rank scratch
    assert fb.fsvd_ffn_workspace(big, 2048, 2048) > fb.FSVD_STATIC_SCRATCH_BYTES
    assert call(big, fac(4096, 2048, 16384), fac(16384, 2048, 4096)) == WORKSPACE
    text = open(os.path.join(ROOT, "include", "fsvd.h")).read()
    assert re.search(r"#define\s+FSVD_STATIC_SCRATCH_BYTES\s+\(\(size_t\)32\s*<<\s*20\)", text)
    assert fb.FSVD_STATIC_SCRATCH_BYTES == 32 << 20


def test_probe_entry_points_validate_their_arguments():
    L = fb.lib()
    assert L.fsvd_mfma_probe(0, 10, 256, None) == INVALID
    assert L.fsvd_mfma_probe(4, 0, 256, None) == INVALID
    assert L.fsvd_mfma_probe(4, 10, None, None) == INVALID
    assert L.fsvd_dma_probe(4, 10, 0, None, 32768, 256, None) == INVALID
    assert L.fsvd_dma_probe(4, 10, 0, 256, 1000, 256, None) == INVALID          # region not a multiple of 32 KiB
    assert L.fsvd_dma_probe(4, 10, 0, 256, 0, 256, None) == INVALID
    assert L.fsvd_dma_probe(0, 10, 0, 256, 32768, 256, None) == INVALID


def test_one_kernel_ffn_contract():
    """fsvd_ffn_v2 takes only tile images of all four matrices and ranks up to 1024, and says so before any launch."""
    L = fb.lib()
    d = desc()

    def lay(f, u=1, v=1):
        return fb.fsvd_factor(f.U, f.V, f.bias, f.in_dim, f.rank, f.out_dim, u, v)
    w1, w2 = fac(768, 64, 3072), fac(3072, 64, 768)
    call = lambda a, b, x=256, out=256: L.fsvd_ffn_v2(C.byref(d), x, C.byref(a), C.byref(b), out, None)
    assert call(lay(w1), lay(w2), x=None) == INVALID                      # valid factors, then X is NULL
    assert call(lay(w1), lay(w2), out=264) == INVALID                     # misaligned result
    assert call(lay(w1, u=0), lay(w2)) == UNSUPPORTED                     # every matrix must be a tile image
    assert call(lay(w1), lay(w2, v=0)) == UNSUPPORTED
    assert call(w1, w2) == UNSUPPORTED
    big1, big2 = fac(768, 1040, 3072), fac(3072, 1040, 768)
    assert call(lay(big1), lay(w2)) == UNSUPPORTED                        # ranks above 1024
    assert call(lay(w1), lay(big2)) == UNSUPPORTED
    assert call(lay(fac(768, 24, 3072)), lay(w2)) == UNSUPPORTED          # rank not a multiple of 16
    assert call(lay(fac(512, 64, 3072)), lay(w2)) == INVALID              # shapes that do not match the descriptor


def test_grouped_head_factors_contract():
    """`groups` of the *_heads entry points: a divisor of H, the same for q, k, v; 0 means one group per head."""
    L = fb.lib()
    d = desc()                                                                  # H = 12
    o = fac(768, 64, 768)
    need = fb.fsvd_attention_heads_workspace(d, 96, 96, 96, 64)

    def grp(g, r=96):
        f = fac(768, r, 768)
        return fb.fsvd_factor(f.U, f.V, f.bias, f.in_dim, f.rank, f.out_dim, 0, 0, g)
    call = lambda a, b, c: L.fsvd_attention_heads(C.byref(d), None, C.byref(a), C.byref(b), C.byref(c), C.byref(o), 256, 256, need, None)
    for g in (0, 1, 2, 3, 4, 6, 12):
        assert call(grp(g), grp(g), grp(g)) == INVALID                          # passes the factor checks, then X is NULL
    ok = lambda a, b, c: L.fsvd_attention_heads(C.byref(d), 256, C.byref(a), C.byref(b), C.byref(c), C.byref(o), 256, 256, 16, None)
    assert ok(grp(4), grp(4), grp(4)) == WORKSPACE                              # valid factors: only the workspace is short
    assert ok(grp(5), grp(5), grp(5)) == INVALID                                # 5 does not divide 12
    assert ok(grp(-1), grp(-1), grp(-1)) == INVALID
    assert ok(grp(4), grp(2), grp(4)) == UNSUPPORTED                            # q, k, v are grouped alike


def test_decode_entry_points_contract():
    """Sizes of the rank-space KV cache and argument validation of the decoding step (no GPU needed)."""
    L = fb.lib()
    assert L.fsvd_decode_kcache_bytes(2, 70, 64) == 2 * 3 * 1 * 4096          # fragment-major [70, 64] per sequence
    assert L.fsvd_decode_kcache_bytes(16, 4096, 1024) == 16 * 4096 * 1024 * 2
    assert L.fsvd_decode_vcache_bytes(2, 70, 96) == 2 * 3 * 3 * 2048          # 3 rank tiles x 3 key tiles of 2 KiB
    assert L.fsvd_decode_vcache_bytes(16, 4096, 1024) == 16 * 4096 * 1024 * 2
    assert L.fsvd_decode_kcache_bytes(2, 70, 48) == 0 and L.fsvd_decode_vcache_bytes(2, 70, 48) == 0
    assert L.fsvd_decode_kcache_bytes(0, 70, 64) == 0
    d = fb.make_desc(16, 4096, 4096, 32, 16, torch.bfloat16)                     # M is the cache capacity
    q = fac(4096, 1024, 4096)
    need = fb.fsvd_decode_attention_workspace(d, 1024, 1024, 1024, 1024)
    assert need > 0 and need % 256 == 0
    # the 2 t r scalars of cache per sequence against the 2 t D of full-width keys and values (appendix, KV-cache cost)
    assert L.fsvd_decode_kcache_bytes(1, 4096, 1024) + L.fsvd_decode_vcache_bytes(1, 4096, 1024) == 2 * 4096 * 1024 * 2
    call = lambda dd, x, kk, kc, tl, ws, n: L.fsvd_decode_attention(C.byref(dd), x, C.byref(q), C.byref(kk), C.byref(q), C.byref(q),
                                                                    kc, 256, tl, 256, ws, n, None)
    assert call(d, None, q, 256, 256, 256, need) == INVALID
    assert call(d, 256, q, None, 256, 256, need) == INVALID
    assert call(d, 256, q, 256, None, 256, need) == INVALID
    assert call(d, 256, q, 256, 256, 256, need - 1) == WORKSPACE
    assert call(d, 256, q, 264, 256, 256, need) == INVALID                      # cache not 16-byte aligned
    assert call(d, 256, fac(4096, 1040, 4096), 256, 256, 256, 1 << 40) == UNSUPPORTED     # r_k % 64
    assert call(d, 256, fac(4096, 2048, 4096), 256, 256, 256, 1 << 40) == UNSUPPORTED     # r_k > 1024
    tiled_v = fb.fsvd_factor(q.U, q.V, q.bias, q.in_dim, q.rank, q.out_dim, 0, 1)
    assert call(d, 256, tiled_v, 256, 256, 256, need) == UNSUPPORTED            # V_k is read row by row here
    assert fb.fsvd_decode_attention_workspace(fb.make_desc(16, 4096, 4096, 64, 16, torch.bfloat16), 1024, 1024, 1024, 1024) == 0   # H > 32
    assert L.fsvd_decode_cache_write(2, 70, 64, 1, None, 256, 0, 256, None) == INVALID
    assert L.fsvd_decode_cache_write(2, 70, 64, 1, 256, 256, 2, 256, None) == INVALID
    assert L.fsvd_decode_cache_write(2, 70, 48, 1, 256, 256, 0, 256, None) == UNSUPPORTED
    cw = fb.fsvd_decode_core_workspace(d, 1024, 1024)
    assert cw > 0 and cw <= need
    assert L.fsvd_decode_attention_core(C.byref(d), 1024, 1024, 256, 256, 256, 256, 256, 256, cw - 1, None) == WORKSPACE
    assert L.fsvd_decode_attention_core(C.byref(d), 1024, 1024, None, 256, 256, 256, 256, 256, cw, None) == INVALID


def test_per_head_attention_entry_point_contract():
    """Workspace of the per-head entry point = packed X / context + P_q | P_k | P_v with H * rank columns each; the same
    validation as the whole-matrix entry point."""
    L = fb.lib()
    up = lambda n: (n + 255) // 256 * 256
    fm = lambda T, K: ((T + 31) // 32) * ((K + 63) // 64) * 4096
    for name in ("ph_bert_base_b16_m512_r32", "ph_bert_base_b16_m1024_r48", "ph_tiny_r16"):
        w = W.get_workload(name)
        d = fb.make_desc(w.B, w.M, w.D, w.H, w.F, torch.float16)
        need = fb.fsvd_attention_heads_workspace(d, w.r_head, w.r_head, w.r_head, w.r_attn)
        assert need == up(fm(w.T, w.D)) + max(3 * up(fm(w.T, w.H * w.r_head)), up(fm(w.T, w.r_attn)))
        # strictly below the same block with Q, K, V materialised beside P
        if w.T >= 1024:
            assert need < w.T * w.D * 2 + 3 * w.T * w.H * w.r_head * 2 + 3 * w.T * w.D * 2
    d = desc()
    q, o = fac(768, 32, 768), fac(768, 192, 768)
    need = fb.fsvd_attention_heads_workspace(d, 32, 32, 32, 192)
    call = lambda X, out, ws, n, qq=q: L.fsvd_attention_heads(C.byref(d), X, C.byref(qq), C.byref(q), C.byref(q), C.byref(o), out, ws, n, None)
    assert call(None, 256, 256, need) == INVALID
    assert call(256, 256, 256, need - 256) == WORKSPACE
    assert call(256, 256, 256, need, fac(768, 24, 768)) == UNSUPPORTED          # rank % 16
    assert call(256, 256, 256, need, fac(768, 32, 512)) == INVALID              # out_dim must be D
    assert fb.fsvd_attention_heads_workspace(desc(H=7), 32, 32, 32, 64) == 0


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(fb, "_lib", None)
    monkeypatch.setattr(fb, "LIB_PATH", "/nonexistent/libfsvd.so")
    with pytest.raises(FileNotFoundError):
        fb.lib()


def test_gelu_tail_polynomial_of_the_kernel_is_erf_accurate():
    """The FFN kernels evaluate erf-GELU as max(x,0) - |x| 2^p(min(|x|,6)); its coefficients, read from the source,
    must reproduce 0.5 x (1 + erf(x / sqrt 2)) (scipy) to 1e-6 when evaluated in float32 as the kernel does."""
    import re
    from scipy.special import erf
    src = open(os.path.join(ROOT, "paper_2508_01506_amd", "csrc", "fsvd_common.h")).read()
    body = re.search(r"kGeluTail\[7\]\s*=\s*\{([^}]*)\}", src).group(1)
    c = [np.float32(v.strip().rstrip("f")) for v in body.split(",")]
    assert len(c) == 7
    x = np.linspace(-12.0, 12.0, 240001).astype(np.float32)
    t = np.minimum(np.abs(x), np.float32(6.0))
    p = np.full_like(t, c[6])
    for k in range(5, -1, -1):
        p = p * t + c[k]
    got = np.maximum(x, np.float32(0)) - np.abs(x) * np.exp2(p).astype(np.float32)
    ref = 0.5 * x.astype(np.float64) * (1.0 + erf(x.astype(np.float64) / np.sqrt(2.0)))
    assert np.abs(got.astype(np.float64) - ref).max() < 1e-6
