"""ctypes binding of libfsvd.so: argument marshalling only.

Every function here has the name of the C entry point it calls (include/fsvd.h)
and does nothing but turn torch tensors into device pointers, allocate the
output and the workspace with torch (device memory plumbing) and check the
returned status.  All arithmetic happens in the library's HIP kernels; there is
no fallback: if the shared library is missing the import of the native handle
raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfsvd.so")

FSVD_F16, FSVD_BF16, FSVD_F32 = 0, 1, 2
ACT = {"gelu_erf": 0, "gelu_tanh": 1, "relu": 2}
NORM = {"none": 0, "post_ln": 1, "pre_ln": 2}
STATUS = {0: "FSVD_OK", 1: "FSVD_ERR_INVALID_ARG", 2: "FSVD_ERR_UNSUPPORTED", 3: "FSVD_ERR_WORKSPACE",
          4: "FSVD_ERR_DEVICE"}
_TORCH2FSVD = {torch.float16: FSVD_F16, torch.bfloat16: FSVD_BF16, torch.float32: FSVD_F32}

EXPORTS = ["fsvd_attention_workspace", "fsvd_ffn_workspace", "fsvd_layer_workspace", "fsvd_attention_check",
           "fsvd_ffn_check", "fsvd_attention", "fsvd_attention_heads", "fsvd_attention_heads_workspace", "fsvd_ffn",
           "fsvd_layer", "fsvd_layer_heads", "fsvd_layer_heads_workspace", "fsvd_linear", "fsvd_attention_core", "fsvd_attention_heads_core",
           "fsvd_ffn_core", "fsvd_ffn_core_workspace", "fsvd_layernorm", "fsvd_status_string", "fsvd_version", "fsvd_fm_bytes", "fsvd_pack_fm",
           "fsvd_unpack_fm", "fsvd_tiled_bytes", "fsvd_pack_tiled", "fsvd_linear_tiled", "fsvd_decode_kcache_bytes",
           "fsvd_decode_vcache_bytes", "fsvd_decode_cache_write", "fsvd_decode_attention_workspace", "fsvd_decode_attention",
           "fsvd_decode_core_workspace", "fsvd_decode_attention_core",
           "fsvd_attention_groups_workspace", "fsvd_layer_groups_workspace", "fsvd_ffn_v2", "fsvd_ffn_static", "fsvd_mfma_probe", "fsvd_dma_probe"]


class FsvdError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {STATUS.get(status, status)}")


class fsvd_factor(C.Structure):
    _fields_ = [("U", C.c_void_p), ("V", C.c_void_p), ("bias", C.c_void_p),
                ("in_dim", C.c_int32), ("rank", C.c_int32), ("out_dim", C.c_int32),
                ("u_layout", C.c_int32), ("v_layout", C.c_int32), ("groups", C.c_int32)]


class fsvd_desc(C.Structure):
    _fields_ = [("B", C.c_int32), ("M", C.c_int32), ("D", C.c_int32), ("H", C.c_int32), ("F", C.c_int32),
                ("io_dtype", C.c_int), ("out_dtype", C.c_int), ("causal", C.c_int32), ("key_len", C.c_void_p),
                ("softmax_scale", C.c_float), ("act", C.c_int), ("norm", C.c_int), ("ln_eps", C.c_float)]


_lib = None


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -m paper_2508_01506_amd.build` "
                                    "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        P, F, D = C.c_void_p, C.POINTER(fsvd_factor), C.POINTER(fsvd_desc)
        i32, sz = C.c_int32, C.c_size_t
        L.fsvd_attention_workspace.restype = sz
        L.fsvd_attention_workspace.argtypes = [D, i32, i32, i32, i32]
        L.fsvd_ffn_workspace.restype = sz
        L.fsvd_ffn_workspace.argtypes = [D, i32, i32]
        L.fsvd_layer_workspace.restype = sz
        L.fsvd_layer_workspace.argtypes = [D, i32, i32, i32, i32, i32, i32]
        L.fsvd_attention_check.restype = C.c_int
        L.fsvd_attention_check.argtypes = [D, F, F, F, F]
        L.fsvd_ffn_check.restype = C.c_int
        L.fsvd_ffn_check.argtypes = [D, F, F]
        L.fsvd_attention.restype = C.c_int
        L.fsvd_attention.argtypes = [D, P, F, F, F, F, P, P, sz, P]
        L.fsvd_attention_heads_workspace.restype = sz
        L.fsvd_attention_heads_workspace.argtypes = [D, i32, i32, i32, i32]
        L.fsvd_attention_groups_workspace.restype = sz
        L.fsvd_attention_groups_workspace.argtypes = [D, i32, i32, i32, i32, i32]
        L.fsvd_layer_groups_workspace.restype = sz
        L.fsvd_layer_groups_workspace.argtypes = [D, i32, i32, i32, i32, i32, i32, i32]
        L.fsvd_attention_heads.restype = C.c_int
        L.fsvd_attention_heads.argtypes = [D, P, F, F, F, F, P, P, sz, P]
        L.fsvd_ffn.restype = C.c_int
        L.fsvd_ffn.argtypes = [D, P, F, F, P, P, sz, P]
        L.fsvd_dma_probe.restype = C.c_int
        L.fsvd_dma_probe.argtypes = [i32, i32, i32, P, sz, P, P]
        L.fsvd_mfma_probe.restype = C.c_int
        L.fsvd_mfma_probe.argtypes = [i32, i32, P, P]
        L.fsvd_ffn_static.restype = C.c_int
        L.fsvd_ffn_static.argtypes = [D, P, F, F, P, P]
        L.fsvd_ffn_v2.restype = C.c_int
        L.fsvd_ffn_v2.argtypes = [D, P, F, F, P, P]
        L.fsvd_layer.restype = C.c_int
        L.fsvd_layer.argtypes = [D, P, F, F, F, F, P, P, F, F, P, P, P, P, sz, P]
        L.fsvd_layer_heads_workspace.restype = sz
        L.fsvd_layer_heads_workspace.argtypes = [D, i32, i32, i32, i32, i32, i32]
        L.fsvd_layer_heads.restype = C.c_int
        L.fsvd_layer_heads.argtypes = [D, P, F, F, F, F, P, P, F, F, P, P, P, P, sz, P]
        L.fsvd_linear.restype = C.c_int
        L.fsvd_linear.argtypes = [i32, i32, i32, P, C.c_int, P, P, C.c_int, P, C.c_int, P, C.c_int, P]
        L.fsvd_linear_tiled.restype = C.c_int
        L.fsvd_linear_tiled.argtypes = [i32, i32, i32, P, C.c_int, P, P, C.c_int, P, C.c_int, P, C.c_int, P]
        L.fsvd_attention_core.restype = C.c_int
        L.fsvd_attention_core.argtypes = [D, P, P, P, F, F, F, P, P]
        L.fsvd_attention_heads_core.restype = C.c_int
        L.fsvd_attention_heads_core.argtypes = [D, P, P, P, F, F, F, P, P]
        L.fsvd_ffn_core_workspace.restype = sz
        L.fsvd_ffn_core_workspace.argtypes = [D, i32, i32]
        L.fsvd_ffn_core.restype = C.c_int
        L.fsvd_ffn_core.argtypes = [D, P, F, F, P, P, sz, P]
        L.fsvd_layernorm.restype = C.c_int
        L.fsvd_layernorm.argtypes = [i32, i32, P, C.c_int, P, P, C.c_int, C.c_float, P, C.c_int, P]
        L.fsvd_fm_bytes.restype = sz
        L.fsvd_fm_bytes.argtypes = [i32, i32]
        L.fsvd_pack_fm.restype = C.c_int
        L.fsvd_pack_fm.argtypes = [i32, i32, P, C.c_int, P, P]
        L.fsvd_unpack_fm.restype = C.c_int
        L.fsvd_unpack_fm.argtypes = [i32, i32, P, P, C.c_int, P]
        L.fsvd_tiled_bytes.restype = sz
        L.fsvd_tiled_bytes.argtypes = [i32, i32]
        L.fsvd_pack_tiled.restype = C.c_int
        L.fsvd_pack_tiled.argtypes = [i32, i32, P, C.c_int, P, P]
        L.fsvd_decode_kcache_bytes.restype = sz
        L.fsvd_decode_kcache_bytes.argtypes = [i32, i32, i32]
        L.fsvd_decode_vcache_bytes.restype = sz
        L.fsvd_decode_vcache_bytes.argtypes = [i32, i32, i32]
        L.fsvd_decode_cache_write.restype = C.c_int
        L.fsvd_decode_cache_write.argtypes = [i32, i32, i32, i32, P, P, i32, P, P]
        L.fsvd_decode_attention_workspace.restype = sz
        L.fsvd_decode_attention_workspace.argtypes = [D, i32, i32, i32, i32]
        L.fsvd_decode_attention.restype = C.c_int
        L.fsvd_decode_attention.argtypes = [D, P, F, F, F, F, P, P, P, P, P, sz, P]
        L.fsvd_decode_core_workspace.restype = sz
        L.fsvd_decode_core_workspace.argtypes = [D, i32, i32]
        L.fsvd_decode_attention_core.restype = C.c_int
        L.fsvd_decode_attention_core.argtypes = [D, i32, i32, P, P, P, P, P, P, sz, P]
        L.fsvd_status_string.restype = C.c_char_p
        L.fsvd_status_string.argtypes = [C.c_int]
        L.fsvd_version.restype = i32
        L.fsvd_version.argtypes = []
        _lib = L
    return _lib


# ---------------------------------------------------------------------------------------------
# marshalling helpers
# ---------------------------------------------------------------------------------------------

@dataclass
class Factor:
    """Device tensors of one factored projection (U [in, r], V [r, out], b [out] or None).

    U_tiled / V_tiled: optional tile images of U / V made by fsvd_pack_tiled (uint8 buffers); when present they are
    what the library is handed, with the matching layout member set to FSVD_TILED."""
    U: torch.Tensor
    V: torch.Tensor
    b: Optional[torch.Tensor] = None
    U_tiled: Optional[torch.Tensor] = None
    V_tiled: Optional[torch.Tensor] = None

    def c(self) -> fsvd_factor:
        for t in (self.U, self.V, self.b, self.U_tiled, self.V_tiled):
            assert t is None or (t.is_contiguous() and t.is_cuda)
        u = self.U if self.U_tiled is None else self.U_tiled
        v = self.V if self.V_tiled is None else self.V_tiled
        return fsvd_factor(u.data_ptr(), v.data_ptr(), 0 if self.b is None else self.b.data_ptr(),
                           self.U.shape[0], self.U.shape[1], self.V.shape[1],
                           int(self.U_tiled is not None), int(self.V_tiled is not None))

    def with_tiled(self, u: bool = False, v: bool = False) -> "Factor":
        """A copy of this factor whose U and / or V are additionally held as tile images."""
        return Factor(self.U, self.V, self.b, fsvd_pack_tiled(self.U) if u else self.U_tiled,
                      fsvd_pack_tiled(self.V) if v else self.V_tiled)

    @property
    def rank(self) -> int:
        return self.U.shape[1]


@dataclass
class HeadFactor(Factor):
    """Per-head or grouped-head factors of one attention projection: U [D, G r], V [G, r, D / G], b [D] or None
    (G = H: one pair per head)."""

    def c(self) -> fsvd_factor:
        for t in (self.U, self.V, self.b):
            assert t is None or (t.is_contiguous() and t.is_cuda)
        G, r, width = self.V.shape
        assert self.U.shape[1] == G * r and self.V_tiled is None
        u = self.U if self.U_tiled is None else self.U_tiled
        return fsvd_factor(u.data_ptr(), self.V.data_ptr(), 0 if self.b is None else self.b.data_ptr(),
                           self.U.shape[0], r, G * width, int(self.U_tiled is not None), 0, G)

    def with_tiled(self, u: bool = False, v: bool = False) -> "HeadFactor":
        assert not v, "V of a per-head factor stays row-major"
        return HeadFactor(self.U, self.V, self.b, fsvd_pack_tiled(self.U) if u else self.U_tiled, None)

    @property
    def rank(self) -> int:
        return self.V.shape[1]


def _ptr(t: Optional[torch.Tensor]) -> int:
    if t is None:
        return 0
    assert t.is_cuda and t.is_contiguous()
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def make_desc(B, M, D, H, F, io_dtype, out_dtype=torch.float32, causal=False, key_len=None, softmax_scale=0.0,
              act="gelu_erf", norm="post_ln", ln_eps=1e-5) -> fsvd_desc:
    if key_len is not None:
        assert key_len.dtype == torch.int32 and key_len.is_cuda and key_len.is_contiguous()
    return fsvd_desc(B, M, D, H, F, _TORCH2FSVD[io_dtype], _TORCH2FSVD[out_dtype], int(bool(causal)),
                     _ptr(key_len), float(softmax_scale), ACT[act], NORM[norm], float(ln_eps))


def _check(status: int, where: str) -> None:
    if status != 0:
        raise FsvdError(status, where)


def _workspace(nbytes: int, device) -> torch.Tensor:
    if nbytes == 0:
        raise FsvdError(2, "workspace size query rejected the configuration")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def _out_dtype(desc: fsvd_desc):
    return {FSVD_F16: torch.float16, FSVD_BF16: torch.bfloat16, FSVD_F32: torch.float32}[desc.out_dtype]


# ---------------------------------------------------------------------------------------------
# entry points (same names as the C ABI)
# ---------------------------------------------------------------------------------------------

def fsvd_attention_workspace(desc, r_q, r_k, r_v, r_o) -> int:
    return lib().fsvd_attention_workspace(C.byref(desc), r_q, r_k, r_v, r_o)


def fsvd_attention_heads_workspace(desc, r_q, r_k, r_v, r_o) -> int:
    return lib().fsvd_attention_heads_workspace(C.byref(desc), r_q, r_k, r_v, r_o)


def fsvd_attention_groups_workspace(desc, groups, r_q, r_k, r_v, r_o) -> int:
    return lib().fsvd_attention_groups_workspace(C.byref(desc), groups, r_q, r_k, r_v, r_o)


def fsvd_attention_heads(desc, X, q: HeadFactor, k: HeadFactor, v: HeadFactor, o: Factor, out=None, workspace=None):
    """Attention block with per-head factors of q, k, v (o: whole-matrix factor)."""
    if out is None:
        out = torch.empty(X.shape, dtype=_out_dtype(desc), device=X.device)
    if workspace is None:
        workspace = _workspace(fsvd_attention_groups_workspace(desc, q.V.shape[0], q.rank, k.rank, v.rank, o.rank), X.device)
    fq, fk, fv, fo = q.c(), k.c(), v.c(), o.c()
    _check(lib().fsvd_attention_heads(C.byref(desc), _ptr(X), C.byref(fq), C.byref(fk), C.byref(fv), C.byref(fo),
                                      _ptr(out), _ptr(workspace), workspace.numel(), _stream()), "fsvd_attention_heads")
    return out


def fsvd_ffn_workspace(desc, r_1, r_2) -> int:
    return lib().fsvd_ffn_workspace(C.byref(desc), r_1, r_2)


def fsvd_layer_workspace(desc, r_q, r_k, r_v, r_o, r_1, r_2) -> int:
    return lib().fsvd_layer_workspace(C.byref(desc), r_q, r_k, r_v, r_o, r_1, r_2)


def fsvd_attention(desc, X, q: Factor, k: Factor, v: Factor, o: Factor, out=None, workspace=None):
    if out is None:
        out = torch.empty(X.shape, dtype=_out_dtype(desc), device=X.device)
    if workspace is None:
        workspace = _workspace(fsvd_attention_workspace(desc, q.rank, k.rank, v.rank, o.rank), X.device)
    fq, fk, fv, fo = q.c(), k.c(), v.c(), o.c()
    _check(lib().fsvd_attention(C.byref(desc), _ptr(X), C.byref(fq), C.byref(fk), C.byref(fv), C.byref(fo),
                                _ptr(out), _ptr(workspace), workspace.numel(), _stream()), "fsvd_attention")
    return out


def fsvd_ffn(desc, X, w1: Factor, w2: Factor, out=None, workspace=None):
    if out is None:
        out = torch.empty(X.shape, dtype=_out_dtype(desc), device=X.device)
    if workspace is None:
        workspace = _workspace(fsvd_ffn_workspace(desc, w1.rank, w2.rank), X.device)
    f1, f2 = w1.c(), w2.c()
    _check(lib().fsvd_ffn(C.byref(desc), _ptr(X), C.byref(f1), C.byref(f2), _ptr(out), _ptr(workspace),
                          workspace.numel(), _stream()), "fsvd_ffn")
    return out


def fsvd_mfma_probe(workgroups: int, iters: int, out):
    """Launch the matrix-core rate probe; returns the FLOP it executes.  out: float32 tensor of workgroups * 256 elements."""
    _check(lib().fsvd_mfma_probe(workgroups, iters, _ptr(out), _stream()), "fsvd_mfma_probe")
    return workgroups * 4 * iters * 4 * 32768


def fsvd_dma_probe(workgroups: int, steps: int, with_work: bool, src, region_bytes: int, out):
    """Launch the L2 -> LDS delivery probe; returns the bytes it moves.  src: 8 * region_bytes bytes; out: float32[workgroups * 512]."""
    assert src.numel() * src.element_size() >= 8 * region_bytes
    _check(lib().fsvd_dma_probe(workgroups, steps, int(with_work), _ptr(src), region_bytes, _ptr(out), _stream()), "fsvd_dma_probe")
    return workgroups * steps * 32768


FSVD_STATIC_SCRATCH_BYTES = 32 << 20


def fsvd_ffn_static(desc, X, w1: Factor, w2: Factor, out):
    """fsvd_ffn with the library's own static scratch instead of a workspace; `out` is the caller's (nothing is allocated)."""
    f1, f2 = w1.c(), w2.c()
    _check(lib().fsvd_ffn_static(C.byref(desc), _ptr(X), C.byref(f1), C.byref(f2), _ptr(out), _stream()), "fsvd_ffn_static")
    return out


def fsvd_ffn_v2(desc, X, w1: Factor, w2: Factor, out=None):
    """The FFN block as one kernel without workspace; both factors need U and V as tile images."""
    if out is None:
        out = torch.empty(X.shape, dtype=_out_dtype(desc), device=X.device)
    f1, f2 = w1.c(), w2.c()
    _check(lib().fsvd_ffn_v2(C.byref(desc), _ptr(X), C.byref(f1), C.byref(f2), _ptr(out), _stream()), "fsvd_ffn_v2")
    return out


def fsvd_layer(desc, X, q, k, v, o, ln1_gamma, ln1_beta, w1, w2, ln2_gamma, ln2_beta, out=None, workspace=None):
    if out is None:
        out = torch.empty(X.shape, dtype=_out_dtype(desc), device=X.device)
    if workspace is None:
        workspace = _workspace(fsvd_layer_workspace(desc, q.rank, k.rank, v.rank, o.rank, w1.rank, w2.rank), X.device)
    fq, fk, fv, fo, f1, f2 = q.c(), k.c(), v.c(), o.c(), w1.c(), w2.c()
    _check(lib().fsvd_layer(C.byref(desc), _ptr(X), C.byref(fq), C.byref(fk), C.byref(fv), C.byref(fo),
                            _ptr(ln1_gamma), _ptr(ln1_beta), C.byref(f1), C.byref(f2), _ptr(ln2_gamma),
                            _ptr(ln2_beta), _ptr(out), _ptr(workspace), workspace.numel(), _stream()), "fsvd_layer")
    return out


def fsvd_layer_heads_workspace(desc, r_q, r_k, r_v, r_o, r_1, r_2) -> int:
    return lib().fsvd_layer_heads_workspace(C.byref(desc), r_q, r_k, r_v, r_o, r_1, r_2)


def fsvd_layer_groups_workspace(desc, groups, r_q, r_k, r_v, r_o, r_1, r_2) -> int:
    return lib().fsvd_layer_groups_workspace(C.byref(desc), groups, r_q, r_k, r_v, r_o, r_1, r_2)


def fsvd_layer_heads(desc, X, q, k, v, o, ln1_gamma, ln1_beta, w1, w2, ln2_gamma, ln2_beta, out=None, workspace=None):
    """One layer with per-head factors of q, k, v (HeadFactor); o, w1, w2 whole-matrix factors."""
    if out is None:
        out = torch.empty(X.shape, dtype=_out_dtype(desc), device=X.device)
    if workspace is None:
        workspace = _workspace(fsvd_layer_groups_workspace(desc, q.V.shape[0], q.rank, k.rank, v.rank, o.rank, w1.rank, w2.rank),
                               X.device)
    fq, fk, fv, fo, f1, f2 = q.c(), k.c(), v.c(), o.c(), w1.c(), w2.c()
    _check(lib().fsvd_layer_heads(C.byref(desc), _ptr(X), C.byref(fq), C.byref(fk), C.byref(fv), C.byref(fo),
                                  _ptr(ln1_gamma), _ptr(ln1_beta), C.byref(f1), C.byref(f2), _ptr(ln2_gamma),
                                  _ptr(ln2_beta), _ptr(out), _ptr(workspace), workspace.numel(), _stream()),
           "fsvd_layer_heads")
    return out


def fsvd_linear(A, W, bias=None, residual=None, out_dtype=torch.float16, out=None):
    T, K = A.shape
    N = W.shape[1]
    if out is None:
        out = torch.empty((T, N), dtype=out_dtype, device=A.device)
    _check(lib().fsvd_linear(T, K, N, _ptr(A), _TORCH2FSVD[A.dtype], _ptr(W), _ptr(bias), _TORCH2FSVD[W.dtype],
                             _ptr(residual), 0 if residual is None else _TORCH2FSVD[residual.dtype], _ptr(out),
                             _TORCH2FSVD[out.dtype], _stream()), "fsvd_linear")
    return out


def fsvd_linear_tiled(A, W_tiled, N, bias=None, residual=None, out_dtype=torch.float16, out=None,
                      bias_dtype=torch.float16):
    """fsvd_linear with the weight given as tile images of [K, N] (fsvd_pack_tiled)."""
    T, K = A.shape
    if out is None:
        out = torch.empty((T, N), dtype=out_dtype, device=A.device)
    bdt = bias.dtype if bias is not None else bias_dtype
    _check(lib().fsvd_linear_tiled(T, K, N, _ptr(A), _TORCH2FSVD[A.dtype], _ptr(W_tiled), _ptr(bias), _TORCH2FSVD[bdt],
                                   _ptr(residual), 0 if residual is None else _TORCH2FSVD[residual.dtype], _ptr(out),
                                   _TORCH2FSVD[out.dtype], _stream()), "fsvd_linear_tiled")
    return out


def fsvd_fm_bytes(T, K) -> int:
    return lib().fsvd_fm_bytes(T, K)


def fsvd_pack_fm(src, out=None):
    """Row-major [T, K] (fp16 / bf16 / fp32) -> fragment-major fp16 buffer (uint8 tensor)."""
    T, K = src.shape
    if out is None:
        out = torch.empty(fsvd_fm_bytes(T, K), dtype=torch.uint8, device=src.device)
    _check(lib().fsvd_pack_fm(T, K, _ptr(src), _TORCH2FSVD[src.dtype], _ptr(out), _stream()), "fsvd_pack_fm")
    return out


def fsvd_tiled_bytes(rows: int, cols: int) -> int:
    return lib().fsvd_tiled_bytes(rows, cols)


def fsvd_pack_tiled(src, out=None):
    """Row-major weight matrix [rows, cols] (fp16 / bf16) -> fp16 tile images (uint8 tensor)."""
    rows, cols = src.shape
    if out is None:
        out = torch.empty(fsvd_tiled_bytes(rows, cols), dtype=torch.uint8, device=src.device)
    _check(lib().fsvd_pack_tiled(rows, cols, _ptr(src), _TORCH2FSVD[src.dtype], _ptr(out), _stream()), "fsvd_pack_tiled")
    return out


def fsvd_unpack_fm(src_fm, T, K, out_dtype=torch.float16, out=None):
    if out is None:
        out = torch.empty((T, K), dtype=out_dtype, device=src_fm.device)
    _check(lib().fsvd_unpack_fm(T, K, _ptr(src_fm), _ptr(out), _TORCH2FSVD[out.dtype], _stream()), "fsvd_unpack_fm")
    return out


def fsvd_attention_core(desc, Pq, Pk, Pv, q: Factor, k: Factor, v: Factor, out=None):
    """Pq, Pk, Pv and the returned context are fragment-major buffers (see fsvd_pack_fm / fsvd_unpack_fm)."""
    if out is None:
        out = torch.empty(fsvd_fm_bytes(desc.B * desc.M, desc.D), dtype=torch.uint8, device=Pq.device)
    fq, fk, fv = q.c(), k.c(), v.c()
    fn = lib().fsvd_attention_heads_core if isinstance(q, HeadFactor) else lib().fsvd_attention_core
    _check(fn(C.byref(desc), _ptr(Pq), _ptr(Pk), _ptr(Pv), C.byref(fq), C.byref(fk), C.byref(fv), _ptr(out), _stream()),
           "fsvd_attention_core")
    return out


def fsvd_ffn_core_workspace(desc, r1, r2) -> int:
    return lib().fsvd_ffn_core_workspace(C.byref(desc), r1, r2)


def fsvd_ffn_core(desc, P1, w1: Factor, w2: Factor, out=None, workspace=None):
    """P1 and the returned Z are fragment-major buffers."""
    if out is None:
        out = torch.empty(fsvd_fm_bytes(desc.B * desc.M, w2.rank), dtype=torch.uint8, device=P1.device)
    need = fsvd_ffn_core_workspace(desc, w1.rank, w2.rank)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=P1.device)
    f1, f2 = w1.c(), w2.c()
    _check(lib().fsvd_ffn_core(C.byref(desc), _ptr(P1), C.byref(f1), C.byref(f2), _ptr(out), _ptr(workspace),
                               0 if workspace is None else workspace.numel(), _stream()), "fsvd_ffn_core")
    return out


def fsvd_layernorm(X, gamma, beta, eps, out_dtype=torch.float32, out=None):
    T, D = X.shape
    if out is None:
        out = torch.empty((T, D), dtype=out_dtype, device=X.device)
    _check(lib().fsvd_layernorm(T, D, _ptr(X), _TORCH2FSVD[X.dtype], _ptr(gamma), _ptr(beta),
                                _TORCH2FSVD[gamma.dtype], float(eps), _ptr(out), _TORCH2FSVD[out.dtype], _stream()),
           "fsvd_layernorm")
    return out


# ---------------------------------------------------------------------------------------------
# workload plumbing: numpy inputs (already rounded to the storage type) -> device tensors
# ---------------------------------------------------------------------------------------------

# which matrices of which projection the library accepts as tile images: name -> (U, V)
TILED_OK = {n: (True, True) for n in ("q", "k", "v", "o", "w1", "w2")}
TILED_OK_HEADS = {n: (True, False) for n in ("q", "k", "v")}          # per-head factors: V [H, r, d_h] stays row-major


# ---------------------------------------------------------------------------------------------
# decoding step against a rank-space KV cache
# ---------------------------------------------------------------------------------------------

def fsvd_decode_new_caches(B: int, t_max: int, r_k: int, r_v: int, device="cuda:0"):
    """Zero-filled K and V caches (uint8 tensors) of the sizes the library asks for."""
    nk, nv = lib().fsvd_decode_kcache_bytes(B, t_max, r_k), lib().fsvd_decode_vcache_bytes(B, t_max, r_v)
    if not nk or not nv:
        raise FsvdError(2, "fsvd_decode_*cache_bytes")
    return (torch.zeros(nk, dtype=torch.uint8, device=device), torch.zeros(nv, dtype=torch.uint8, device=device))


def fsvd_decode_cache_write(cache, which: int, t_max: int, P_new, t_start):
    """P_new [B, n_new, r] fp16 -> positions t_start[b].. of the K (which = 0) or V (which = 1) cache."""
    B, n_new, r = P_new.shape
    assert P_new.dtype == torch.float16 and t_start.dtype == torch.int32
    _check(lib().fsvd_decode_cache_write(B, t_max, r, n_new, _ptr(t_start), _ptr(P_new), which, _ptr(cache), _stream()),
           "fsvd_decode_cache_write")


def fsvd_decode_attention_workspace(desc, r_q, r_k, r_v, r_o) -> int:
    return lib().fsvd_decode_attention_workspace(C.byref(desc), r_q, r_k, r_v, r_o)


def fsvd_decode_attention(desc, x_new, q: Factor, k: Factor, v: Factor, o: Factor, kcache, vcache, t_len, out=None,
                          workspace=None):
    """One decoding step: x_new [B, D], t_len int32 [B] (tokens already cached) -> out [B, D]; appends to the caches."""
    if out is None:
        out = torch.empty((desc.B, desc.D), dtype=_out_dtype(desc), device=x_new.device)
    if workspace is None:
        workspace = _workspace(fsvd_decode_attention_workspace(desc, q.rank, k.rank, v.rank, o.rank), x_new.device)
    fq, fk, fv, fo = q.c(), k.c(), v.c(), o.c()
    _check(lib().fsvd_decode_attention(C.byref(desc), _ptr(x_new), C.byref(fq), C.byref(fk), C.byref(fv), C.byref(fo),
                                       _ptr(kcache), _ptr(vcache), _ptr(t_len), _ptr(out), _ptr(workspace),
                                       workspace.numel(), _stream()), "fsvd_decode_attention")
    return out


def fsvd_decode_core_workspace(desc, r_k, r_v) -> int:
    return lib().fsvd_decode_core_workspace(C.byref(desc), r_k, r_v)


def fsvd_decode_attention_core(desc, r_k, r_v, W, kcache, vcache, n_keys, out=None, workspace=None):
    """The pass over the cache alone: absorbed queries W (fragment-major [32, r_k] per sequence) -> u [B, H, r_v] fp32."""
    if out is None:
        out = torch.empty((desc.B, desc.H, r_v), dtype=torch.float32, device=W.device)
    if workspace is None:
        workspace = _workspace(fsvd_decode_core_workspace(desc, r_k, r_v), W.device)
    _check(lib().fsvd_decode_attention_core(C.byref(desc), r_k, r_v, _ptr(W), _ptr(kcache), _ptr(vcache), _ptr(n_keys),
                                            _ptr(out), _ptr(workspace), workspace.numel(), _stream()),
           "fsvd_decode_attention_core")
    return out


def to_device(inp: dict, device="cuda:0", tiled: bool = False):
    """Upload the arrays of workloads.make_inputs() in the workload's storage type.  tiled: additionally prepack
    every matrix the library accepts in that form (fsvd_pack_tiled) and hand the library the tile images."""
    w = inp["workload"]
    dt = torch.float16 if w.dtype == "fp16" else torch.bfloat16
    up = lambda a: torch.from_numpy(a).to(device=device, dtype=dt).contiguous()
    dev = {"X": up(inp["X"])}
    for n in ("q", "k", "v", "o", "w1", "w2"):
        cls = HeadFactor if (w.r_head > 0 and n in "qkv") else Factor
        dev[n] = cls(up(inp[n]["U"]), up(inp[n]["V"]), up(inp[n]["b"]))
        if tiled:
            dev[n] = dev[n].with_tiled(*(TILED_OK_HEADS if cls is HeadFactor else TILED_OK)[n])
    for n in ("ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta"):
        dev[n] = up(inp[n])
    dev["key_len"] = None if inp["key_len"] is None else torch.from_numpy(inp["key_len"]).to(device)
    dev["desc"] = make_desc(w.B, w.M, w.D, w.H, w.F, dt, torch.float32, inp["causal"], dev["key_len"], 0.0,
                            "gelu_erf", w.norm, w.ln_eps)
    return dev
