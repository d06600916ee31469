"""Thin Python binding of libff's C ABI (include/ff.h): argument marshalling only.

Every step of the attention path runs inside the HIP library; torch is used here for
device memory and the current stream.  If the library has not been built the import of
any entry point fails loudly - there is no CPU or PyTorch fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG, "libff.so")

FF_OK, FF_EINVAL, FF_EUNSUPPORTED, FF_EWORKSPACE, FF_EHIP = range(5)
FF_F32, FF_BF16 = 0, 1
FF_MSA_ROW, FF_MSA_COL, FF_TRI_START, FF_TRI_END = range(4)

WEIGHT_FIELDS = ("ln_g", "ln_b", "lnz_g", "lnz_b", "w_q", "w_k", "w_v", "w_b", "w_g", "b_g", "w_o", "b_o")


class AttnDesc(C.Structure):
    _fields_ = [("mode", C.c_int32), ("dtype", C.c_int32), ("n_a", C.c_int32), ("n_b", C.c_int32),
                ("c", C.c_int32), ("c_z", C.c_int32), ("heads", C.c_int32), ("head_dim", C.c_int32),
                ("ln_eps", C.c_float)]


class AttnWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_FIELDS]


TRIMUL_FIELDS = ("ln_g", "ln_b", "w_ap", "b_ap", "w_ag", "b_ag", "w_bp", "b_bp", "w_bg", "b_bg", "w_g", "b_g",
                 "lno_g", "lno_b", "w_o", "b_o")


class TriMulDesc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("incoming", C.c_int32), ("n", C.c_int32), ("c_z", C.c_int32), ("c", C.c_int32),
                ("ln_eps", C.c_float)]


class TriMulWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in TRIMUL_FIELDS]


GLOBAL_FIELDS = ("ln_g", "ln_b", "w_q", "w_k", "w_v", "w_g", "b_g", "w_o", "b_o")


class GlobalDesc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("n_seq", C.c_int32), ("n_res", C.c_int32), ("c", C.c_int32), ("heads", C.c_int32),
                ("head_dim", C.c_int32), ("ln_eps", C.c_float)]


class GlobalWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in GLOBAL_FIELDS]


class CoreDesc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("rows", C.c_int32), ("heads", C.c_int32), ("length", C.c_int32), ("head_dim", C.c_int32)]


class FFError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"libff status {status}: {message}")
        self.status = status


_lib = None


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2203_00854_amd.build` "
                "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        L.ff_layernorm.restype = C.c_int
        L.ff_layernorm.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32,
                                   C.c_float, C.c_int32, C.c_void_p]
        L.ff_attention_workspace_bytes.restype = C.c_size_t
        L.ff_attention_workspace_bytes.argtypes = [C.POINTER(AttnDesc), C.c_int32]
        common = [C.POINTER(AttnDesc), C.POINTER(AttnWeights), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                  C.c_void_p, C.c_size_t, C.c_void_p]
        L.ff_gated_attention.restype = C.c_int
        L.ff_gated_attention.argtypes = common
        L.ff_attention_chunked.restype = C.c_int
        L.ff_attention_chunked.argtypes = common + [C.c_int32]
        L.ff_gated_attention_residual.restype = C.c_int
        L.ff_gated_attention_residual.argtypes = common + [C.c_int32]
        L.ff_gated_attention_static.restype = C.c_int
        L.ff_gated_attention_static.argtypes = [C.POINTER(AttnDesc), C.POINTER(AttnWeights), C.c_void_p, C.c_void_p,
                                                C.c_void_p, C.c_void_p, C.c_void_p]
        L.ff_static_scratch_bytes.restype = C.c_size_t
        L.ff_static_scratch_bytes.argtypes = []
        L.ff_triangle_multiplication_workspace_bytes.restype = C.c_size_t
        L.ff_triangle_multiplication_workspace_bytes.argtypes = [C.POINTER(TriMulDesc)]
        L.ff_triangle_multiplication.restype = C.c_int
        L.ff_triangle_multiplication.argtypes = [C.POINTER(TriMulDesc), C.POINTER(TriMulWeights), C.c_void_p, C.c_void_p,
                                                 C.c_void_p, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
        L.ff_global_column_attention_workspace_bytes.restype = C.c_size_t
        L.ff_global_column_attention_workspace_bytes.argtypes = [C.POINTER(GlobalDesc)]
        L.ff_global_column_attention.restype = C.c_int
        L.ff_global_column_attention.argtypes = [C.POINTER(GlobalDesc), C.POINTER(GlobalWeights), C.c_void_p, C.c_void_p,
                                                 C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.ff_attention_core_backward_workspace_bytes.restype = C.c_size_t
        L.ff_attention_core_backward_workspace_bytes.argtypes = [C.POINTER(CoreDesc)]
        L.ff_attention_core_backward.restype = C.c_int
        L.ff_attention_core_backward.argtypes = [C.POINTER(CoreDesc)] + [C.c_void_p] * 13 + [C.c_size_t, C.c_void_p]
        L.ff_attention_path.restype = C.c_char_p
        L.ff_attention_path.argtypes = [C.POINTER(AttnDesc)]
        L.ff_attention_last_path.restype = C.c_char_p
        L.ff_attention_last_path.argtypes = []
        L.ff_profile_enable.restype = None
        L.ff_profile_enable.argtypes = [C.c_int32]
        L.ff_profile_kinds.restype = C.c_int32
        L.ff_profile_name.restype = C.c_char_p
        L.ff_profile_name.argtypes = [C.c_int32]
        L.ff_profile_collect.restype = C.c_int
        L.ff_profile_collect.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        L.ff_probe_sink_bytes.restype = C.c_size_t
        L.ff_probe_sink_bytes.argtypes = []
        L.ff_probe_mfma.restype = C.c_int
        L.ff_probe_mfma.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_double), C.c_void_p]
        L.ff_probe_valu.restype = C.c_int
        L.ff_probe_valu.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_double), C.c_void_p]
        L.ff_probe_copy.restype = C.c_int
        L.ff_probe_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.ff_last_error.restype = C.c_char_p
        L.ff_version.restype = C.c_char_p
        _lib = L
    return _lib


def last_error() -> str:
    return lib().ff_last_error().decode()


def _check(status: int):
    if status != FF_OK:
        raise FFError(status, last_error())


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return FF_F32
    if t.dtype == torch.bfloat16:
        return FF_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def make_desc(mode: int, x, heads: int, head_dim: int, c_z: int = 0, ln_eps: float = 1e-5) -> AttnDesc:
    n_a, n_b, c = x.shape
    return AttnDesc(mode, _dtype_code(x), n_a, n_b, c, c_z, heads, head_dim, ln_eps)


def make_weights(w: Dict[str, "object"]) -> AttnWeights:
    s = AttnWeights()
    for n in WEIGHT_FIELDS:
        t = w.get(n)
        if t is not None:
            assert t.is_contiguous() and t.is_cuda
        setattr(s, n, _ptr(t))
    return s


def ff_layernorm(x, gamma, beta, eps: float = 1e-5, out=None):
    """LayerNorm over the last axis of a contiguous CUDA tensor."""
    import torch
    assert x.is_cuda and x.is_contiguous()
    if out is None:
        out = torch.empty_like(x)
    c = x.shape[-1]
    rows = x.numel() // c if c else 0
    _check(lib().ff_layernorm(_ptr(x), _ptr(gamma), _ptr(beta), _ptr(out), rows, c, eps, _dtype_code(x), _stream()))
    return out


def ff_attention_workspace_bytes(desc: AttnDesc, chunk_rows: int = 0) -> int:
    n = lib().ff_attention_workspace_bytes(C.byref(desc), chunk_rows)
    if n == 0:
        raise FFError(FF_EINVAL, last_error())
    return n


def ff_attention_path(desc: AttnDesc) -> str:
    p = lib().ff_attention_path(C.byref(desc))
    if p is None:
        raise FFError(FF_EINVAL, last_error())
    return p.decode()


def ff_attention_last_path() -> str:
    """Kernel family the last attention call on this thread really launched."""
    return lib().ff_attention_last_path().decode()


def _alloc_ws(nbytes: int, device):
    import torch
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def ff_gated_attention(desc: AttnDesc, w: Dict[str, "object"], x, z=None, mask=None, out=None, ws=None):
    """One gated attention module; returns out [n_a, n_b, c]."""
    import torch
    assert x.is_cuda and x.is_contiguous()
    if out is None:
        out = torch.empty_like(x)
    if ws is None:
        ws = _alloc_ws(ff_attention_workspace_bytes(desc, 0), x.device)
    wts = make_weights(w)
    _check(lib().ff_gated_attention(C.byref(desc), C.byref(wts), _ptr(x), _ptr(z), _ptr(mask), _ptr(out), _ptr(ws),
                                    ws.numel(), _stream()))
    return out


def ff_attention_chunked(desc: AttnDesc, w: Dict[str, "object"], x, z=None, mask=None, chunk_rows: int = 64,
                         out=None, ws=None):
    """The same module, chunk_rows batch rows at a time."""
    import torch
    assert x.is_cuda and x.is_contiguous()
    if out is None:
        out = torch.empty_like(x)
    if ws is None:
        ws = _alloc_ws(ff_attention_workspace_bytes(desc, max(chunk_rows, 1)), x.device)
    wts = make_weights(w)
    _check(lib().ff_attention_chunked(C.byref(desc), C.byref(wts), _ptr(x), _ptr(z), _ptr(mask), _ptr(out), _ptr(ws),
                                      ws.numel(), _stream(), chunk_rows))
    return out


def ff_gated_attention_static(desc: AttnDesc, w: Dict[str, "object"], x, z=None, mask=None, out=None):
    """The module with the library's own device array as workspace: the call itself allocates
    nothing (pass `out`, or this wrapper allocates the result tensor before the call)."""
    import torch
    assert x.is_cuda and x.is_contiguous()
    if out is None:
        out = torch.empty_like(x)
    wts = make_weights(w)
    _check(lib().ff_gated_attention_static(C.byref(desc), C.byref(wts), _ptr(x), _ptr(z), _ptr(mask), _ptr(out),
                                           _stream()))
    return out


def ff_static_scratch_bytes() -> int:
    return lib().ff_static_scratch_bytes()


def ff_triangle_multiplication_workspace_bytes(desc: TriMulDesc) -> int:
    n = lib().ff_triangle_multiplication_workspace_bytes(C.byref(desc))
    if n == 0:
        raise FFError(FF_EINVAL, last_error())
    return n


def ff_triangle_multiplication(desc: TriMulDesc, w: Dict[str, "object"], z, mask=None, residual: bool = False,
                               out=None, ws=None, in_place: bool = False):
    """Triangular multiplicative update of the pair representation z [n, n, c_z]; returns out."""
    import torch
    assert z.is_cuda and z.is_contiguous()
    if in_place:
        out = z
    elif out is None:
        out = torch.empty_like(z)
    if ws is None:
        ws = _alloc_ws(ff_triangle_multiplication_workspace_bytes(desc), z.device)
    wts = TriMulWeights()
    for n in TRIMUL_FIELDS:
        t = w[n]
        assert t.is_contiguous() and t.is_cuda
        setattr(wts, n, _ptr(t))
    _check(lib().ff_triangle_multiplication(C.byref(desc), C.byref(wts), _ptr(z), _ptr(mask), _ptr(out),
                                            1 if residual else 0, _ptr(ws), ws.numel(), _stream()))
    return out


def ff_global_column_attention_workspace_bytes(desc: GlobalDesc) -> int:
    n = lib().ff_global_column_attention_workspace_bytes(C.byref(desc))
    if n == 0:
        raise FFError(FF_EINVAL, last_error())
    return n


def ff_global_column_attention(desc: GlobalDesc, w: Dict[str, "object"], m, mask=None, out=None, ws=None):
    """Global column attention of the extra-MSA stack; m [n_seq, n_res, c]; returns out."""
    import torch
    assert m.is_cuda and m.is_contiguous()
    if out is None:
        out = torch.empty_like(m)
    if ws is None:
        ws = _alloc_ws(ff_global_column_attention_workspace_bytes(desc), m.device)
    wts = GlobalWeights()
    for n in GLOBAL_FIELDS:
        t = w[n]
        assert t.is_contiguous() and t.is_cuda
        setattr(wts, n, _ptr(t))
    _check(lib().ff_global_column_attention(C.byref(desc), C.byref(wts), _ptr(m), _ptr(mask), _ptr(out), _ptr(ws),
                                            ws.numel(), _stream()))
    return out


def ff_attention_core_backward_workspace_bytes(desc: CoreDesc) -> int:
    n = lib().ff_attention_core_backward_workspace_bytes(C.byref(desc))
    if n == 0:
        raise FFError(FF_EINVAL, last_error())
    return n


def ff_attention_core_backward(desc: CoreDesc, q, k, v, g, bias, mask, dout, ws=None):
    """Gradients of the fused attention core; returns (dq, dk, dv, dg, dbias) (dbias None without a bias)."""
    import torch
    for t in (q, k, v, g, dout):
        assert t.is_cuda and t.is_contiguous()
    dq, dk, dv, dg = (torch.empty_like(q) for _ in range(4))
    dbias = None if bias is None else torch.empty_like(bias)
    if ws is None:
        ws = _alloc_ws(ff_attention_core_backward_workspace_bytes(desc), q.device)
    _check(lib().ff_attention_core_backward(C.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(g), _ptr(bias), _ptr(mask),
                                            _ptr(dout), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(dg), _ptr(dbias), _ptr(ws),
                                            ws.numel(), _stream()))
    return dq, dk, dv, dg, dbias


def ff_gated_attention_residual(desc: AttnDesc, w: Dict[str, "object"], x, z=None, mask=None, chunk_rows: int = 0,
                                out=None, ws=None, in_place: bool = False):
    """x + module(x); chunk_rows = 0 takes all batch rows at once.  in_place=True updates x itself."""
    import torch
    assert x.is_cuda and x.is_contiguous()
    if in_place:
        out = x
    elif out is None:
        out = torch.empty_like(x)
    if ws is None:
        ws = _alloc_ws(ff_attention_workspace_bytes(desc, max(chunk_rows, 0)), x.device)
    wts = make_weights(w)
    _check(lib().ff_gated_attention_residual(C.byref(desc), C.byref(wts), _ptr(x), _ptr(z), _ptr(mask), _ptr(out),
                                             _ptr(ws), ws.numel(), _stream(), chunk_rows))
    return out


def ff_profile_enable(on: bool):
    lib().ff_profile_enable(1 if on else 0)


def ff_profile_collect():
    """{kernel kind name: (total milliseconds, launches)} since the timer was switched on."""
    n = lib().ff_profile_kinds()
    ms = (C.c_double * n)()
    cnt = (C.c_int64 * n)()
    _check(lib().ff_profile_collect(ms, cnt))
    return {lib().ff_profile_name(i).decode(): (ms[i], cnt[i]) for i in range(n) if cnt[i]}


def ff_probe_mfma(sink, iters: int) -> float:
    """Enqueue the matrix-instruction probe; returns the flop of the launch."""
    flop = C.c_double(0.0)
    assert sink.numel() * sink.element_size() >= lib().ff_probe_sink_bytes()
    _check(lib().ff_probe_mfma(_ptr(sink), iters, C.byref(flop), _stream()))
    return flop.value


def ff_probe_valu(sink, kind: int, iters: int) -> float:
    """Enqueue the vector-instruction probe of one kind; returns the wavefront-wide instructions of the launch."""
    n = C.c_double(0.0)
    assert sink.numel() * sink.element_size() >= lib().ff_probe_sink_bytes()
    _check(lib().ff_probe_valu(_ptr(sink), kind, iters, C.byref(n), _stream()))
    return n.value


def ff_probe_copy(dst, src):
    """Enqueue the copy probe over the whole of two equally sized contiguous tensors."""
    n = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == n
    _check(lib().ff_probe_copy(_ptr(dst), _ptr(src), n, _stream()))


# ------------------------------------------------------------------------- test/bench glue
def _upload(a, device):
    import numpy as np
    import torch
    if a is None:
        return None
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


def trimul_to_device(case, device="cuda:0"):
    """Upload a seeded triangular-update case (inputs.TriMulCase).  Returns (desc, weights, z, mask)."""
    sp = case.spec
    desc = TriMulDesc(FF_F32 if sp.dtype == "f32" else FF_BF16, 1 if sp.incoming else 0, sp.n, sp.c_z, sp.c, sp.ln_eps)
    return desc, {k: _upload(v, device) for k, v in case.weights.items()}, _upload(case.z, device), _upload(case.mask, device)


def global_to_device(case, device="cuda:0"):
    """Upload a seeded global-column-attention case (inputs.GlobalCase).  Returns (desc, weights, m, mask)."""
    sp = case.spec
    desc = GlobalDesc(FF_F32 if sp.dtype == "f32" else FF_BF16, sp.n_seq, sp.n_res, sp.c, sp.heads, sp.head_dim, sp.ln_eps)
    return desc, {k: _upload(v, device) for k, v in case.weights.items()}, _upload(case.m, device), _upload(case.mask, device)


def core_to_device(case, device="cuda:0"):
    """Upload a seeded attention-core case (inputs.CoreCase).  Returns (desc, tensors dict, mask)."""
    sp = case.spec
    desc = CoreDesc(FF_BF16, sp.rows, sp.heads, sp.length, sp.head_dim)
    return desc, {k: _upload(v, device) for k, v in case.tensors.items()}, _upload(case.mask, device)


def to_device(case, device="cuda:0"):
    """Upload a seeded case (paper_2203_00854_amd.inputs.Case) as torch tensors.
    Returns (desc, weights, x, z, mask)."""
    import numpy as np
    import torch

    def up(a):
        if a is None:
            return None
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
        return torch.from_numpy(a).to(device)

    sp = case.spec
    x = up(case.x)
    z = up(case.z)
    mask = up(case.mask)
    w = {k: up(v) for k, v in case.weights.items()}
    desc = AttnDesc(sp.mode, FF_F32 if sp.dtype == "f32" else FF_BF16, sp.n_a, sp.n_b, sp.c, sp.c_z, sp.heads,
                    sp.head_dim, sp.ln_eps)
    return desc, w, x, z, mask
