"""ctypes binding of libpskv.so: same names as include/pskv.h, argument marshalling only.

Every step of the attention path runs inside the HIP library.  There is no fallback: if the
library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
# PSKV_LIB: another build of the library to load instead of the in-tree one (kernel experiments)
LIB_PATH = os.environ.get("PSKV_LIB") or os.path.join(HERE, "libpskv.so")

PSKV_OK, PSKV_ERR_INVALID_ARG, PSKV_ERR_UNSUPPORTED, PSKV_ERR_WORKSPACE, PSKV_ERR_HIP = range(5)
PSKV_DTYPE_F32, PSKV_DTYPE_BF16 = 0, 1
PSKV_IMPL_AUTO, PSKV_IMPL_SIMPLE, PSKV_IMPL_MFMA = 0, 1, 2
_IMPL = {"auto": PSKV_IMPL_AUTO, "simple": PSKV_IMPL_SIMPLE, "mfma": PSKV_IMPL_MFMA}

EXPORTS = ["pskv_version", "pskv_status_str", "pskv_last_error", "pskv_attn_fwd_workspace_bytes",
           "pskv_attn_validate", "pskv_attn_fwd",
           "pskv_attn_multi_validate", "pskv_attn_fwd_multi", "pskv_attn_bwd", "pskv_attn_bwd_multi",
           "pskv_attn_bwd_workspace_bytes", "pskv_attn_bwd_noalloc"]
PSKV_NOALLOC_SCRATCH_BYTES = 8 << 20


class pskv_attn_params(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("B", "S", "P", "Hq", "Hkv", "D", "dtype", "impl")] + \
               [("scale", ctypes.c_float), ("reserved", ctypes.c_int32)] + \
               [(n, ctypes.c_int64) for n in (
                   "q_stride_b", "q_stride_s", "q_stride_h",
                   "ks_stride_b", "ks_stride_s", "ks_stride_h",
                   "kp_stride_p", "kp_stride_h",
                   "o_stride_b", "o_stride_s", "o_stride_h")]


class pskv_multi_params(ctypes.Structure):
    _fields_ = [("base", pskv_attn_params), ("Np", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("kp_stride_n", ctypes.c_int64)]


class PskvError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"pskv status {status} ({what})")
        self.status = status


_lib = None


def load():
    """Load the built library; raise if it is missing (no CPU or PyTorch fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with __graft_entry__.build() "
                          "or `python -m paper_2603_13420_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    P = ctypes.POINTER(pskv_attn_params)
    vp = ctypes.c_void_p
    lib.pskv_version.restype = ctypes.c_int
    lib.pskv_status_str.restype = ctypes.c_char_p
    lib.pskv_status_str.argtypes = [ctypes.c_int]
    lib.pskv_last_error.restype = ctypes.c_char_p
    lib.pskv_attn_fwd_workspace_bytes.restype = ctypes.c_size_t
    lib.pskv_attn_fwd_workspace_bytes.argtypes = [P]
    lib.pskv_attn_validate.restype = ctypes.c_int
    lib.pskv_attn_validate.argtypes = [P]
    fwd_args = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.pskv_attn_fwd.restype = ctypes.c_int
    lib.pskv_attn_fwd.argtypes = fwd_args
    PM = ctypes.POINTER(pskv_multi_params)
    lib.pskv_attn_multi_validate.restype = ctypes.c_int
    lib.pskv_attn_multi_validate.argtypes = [PM]
    lib.pskv_attn_fwd_multi.restype = ctypes.c_int
    lib.pskv_attn_fwd_multi.argtypes = [PM, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.pskv_attn_bwd.restype = ctypes.c_int
    lib.pskv_attn_bwd.argtypes = [P] + [vp] * 13 + [ctypes.c_size_t, vp]
    lib.pskv_attn_bwd_workspace_bytes.restype = ctypes.c_size_t
    lib.pskv_attn_bwd_workspace_bytes.argtypes = [P]
    lib.pskv_attn_bwd_multi.restype = ctypes.c_int
    lib.pskv_attn_bwd_multi.argtypes = [PM] + [vp] * 14 + [ctypes.c_size_t, vp]
    lib.pskv_attn_bwd_noalloc.restype = ctypes.c_int
    lib.pskv_attn_bwd_noalloc.argtypes = [P] + [vp] * 13
    _lib = lib
    return lib


def pskv_version() -> int:
    return int(load().pskv_version())


def pskv_status_str(status: int) -> str:
    return load().pskv_status_str(int(status)).decode()


def pskv_last_error() -> str:
    return load().pskv_last_error().decode()


def _raise(status: int):
    raise PskvError(status, f"{pskv_status_str(status)}: {pskv_last_error()}")


def make_params(B, S, P, Hq, Hkv, D, dtype: str, impl: str = "auto", scale: float = 0.0,
                **strides) -> pskv_attn_params:
    p = pskv_attn_params()
    p.B, p.S, p.P, p.Hq, p.Hkv, p.D = B, S, P, Hq, Hkv, D
    p.dtype = {"f32": PSKV_DTYPE_F32, "bf16": PSKV_DTYPE_BF16}[dtype]
    p.impl = _IMPL[impl]
    p.scale = scale
    p.reserved = 0
    for k, v in strides.items():
        setattr(p, k, int(v))
    return p


def pskv_attn_validate(p: pskv_attn_params) -> int:
    return int(load().pskv_attn_validate(ctypes.byref(p)))


def pskv_attn_fwd_workspace_bytes(p: pskv_attn_params) -> int:
    n = int(load().pskv_attn_fwd_workspace_bytes(ctypes.byref(p)))
    if n == ctypes.c_size_t(-1).value:
        _raise(pskv_attn_validate(p))
    return n


def _stride(t, dim: int, name: str) -> int:
    """Element stride of dimension `dim` as the C ABI wants it.  The ABI reads 0 as "contiguous", so
    a real stride of 0 (an expanded view, e.g. one prefix broadcast over the instructions) must not
    reach it: the kernels would run over the end of the allocation.  A dimension of size 1 has no
    stride to speak of and is passed as 0."""
    if t.shape[dim] <= 1:
        return 0
    if t.stride(dim) == 0:
        raise ValueError(f"{name}: dimension {dim} of size {t.shape[dim]} has stride 0 (an expanded view); "
                         "materialise it with .contiguous()")
    return t.stride(dim)


def _params_from_tensors(q, k_suf, k_pre, out, impl, scale):
    import torch
    B, S, Hq, D = q.shape
    Hkv = k_suf.shape[2]
    P = 0 if k_pre is None else k_pre.shape[0]
    dtype = {torch.float32: "f32", torch.bfloat16: "bf16"}[q.dtype]
    for t in (q, k_suf, out) + (() if k_pre is None else (k_pre,)):
        if t.shape[-1] > 1 and t.stride(-1) != 1:
            raise ValueError("innermost dimension must have stride 1")
    st = dict(q_stride_b=_stride(q, 0, "q"), q_stride_s=_stride(q, 1, "q"), q_stride_h=_stride(q, 2, "q"),
              ks_stride_b=_stride(k_suf, 0, "k_suf"), ks_stride_s=_stride(k_suf, 1, "k_suf"),
              ks_stride_h=_stride(k_suf, 2, "k_suf"),
              o_stride_b=_stride(out, 0, "out"), o_stride_s=_stride(out, 1, "out"), o_stride_h=_stride(out, 2, "out"))
    if k_pre is not None and P > 0:
        st.update(kp_stride_p=_stride(k_pre, 0, "k_pre"), kp_stride_h=_stride(k_pre, 1, "k_pre"))
    return make_params(B, S, P, Hq, Hkv, D, dtype, impl, scale, **st)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _check_inputs(q, k_suf, v_suf, k_pre, v_pre, suf_len, out, lse):
    import torch
    dev = q.device
    if dev.type != "cuda":
        raise ValueError("tensors must live on the GPU")
    for name, t in (("k_suf", k_suf), ("v_suf", v_suf), ("k_pre", k_pre), ("v_pre", v_pre), ("out", out)):
        if t is None:
            continue
        if t.device != dev or t.dtype != q.dtype:
            raise ValueError(f"{name}: device/dtype differ from q")
    B, S, Hq, D = q.shape
    Hkv = k_suf.shape[2]
    if tuple(k_suf.shape) != (B, S, Hkv, D) or tuple(v_suf.shape) != (B, S, Hkv, D):
        raise ValueError("k_suf/v_suf must be [B,S,Hkv,D]")
    if v_suf.stride() != k_suf.stride():
        raise ValueError("k_suf and v_suf must share strides")
    if k_pre is not None:
        if tuple(k_pre.shape[1:]) != (Hkv, D) or tuple(v_pre.shape) != tuple(k_pre.shape):
            raise ValueError("k_pre/v_pre must be [P,Hkv,D]")
        if v_pre.stride() != k_pre.stride():
            raise ValueError("k_pre and v_pre must share strides")
    if tuple(out.shape) != (B, S, Hq, D):
        raise ValueError("out must be [B,S,Hq,D]")
    if suf_len is not None and (suf_len.dtype != torch.int32 or tuple(suf_len.shape) != (B,)
                                or not suf_len.is_contiguous() or suf_len.device != dev):
        raise ValueError("suf_len must be a contiguous int32 [B] tensor on the same device")
    if lse is not None and (lse.dtype != torch.float32 or tuple(lse.shape) != (B, Hq, S)
                            or not lse.is_contiguous() or lse.device != dev):
        raise ValueError("lse must be a contiguous float32 [B,Hq,S] tensor on the same device")


def pskv_attn_fwd(q, k_suf, v_suf, k_pre, v_pre, suf_len=None, out=None, lse=None,
                  impl: str = "auto", scale: float = 0.0, stream: Optional[int] = None):
    """Enqueue one forward call on torch's current stream (or `stream`, a raw hipStream_t).
    `out` (and `lse`) are allocated by torch when not given; returns `out`."""
    import torch
    if out is None:
        out = torch.empty_like(q)
    _check_inputs(q, k_suf, v_suf, k_pre, v_pre, suf_len, out, lse)
    p = _params_from_tensors(q, k_suf, k_pre, out, impl, scale)
    if stream is None:
        stream = torch.cuda.current_stream(q.device).cuda_stream
    with torch.cuda.device(q.device):
        rc = load().pskv_attn_fwd(ctypes.byref(p), _ptr(q), _ptr(k_suf), _ptr(v_suf), _ptr(k_pre),
                                  _ptr(v_pre), _ptr(suf_len), _ptr(out), _ptr(lse), None, 0,
                                  ctypes.c_void_p(stream))
    if rc != PSKV_OK:
        _raise(rc)
    return out


class PreparedCall:
    """pskv_attn_fwd with every argument marshalled once: calling it costs one foreign call.
    The tensors must stay alive and unmoved for as long as the object is used."""

    def __init__(self, q, k_suf, v_suf, k_pre, v_pre, suf_len, out, lse=None, impl: str = "auto",
                 scale: float = 0.0, stream: Optional[int] = None):
        import torch
        _check_inputs(q, k_suf, v_suf, k_pre, v_pre, suf_len, out, lse)
        self._keep = (q, k_suf, v_suf, k_pre, v_pre, suf_len, out, lse)
        self._p = _params_from_tensors(q, k_suf, k_pre, out, impl, scale)
        if stream is None:
            stream = torch.cuda.current_stream(q.device).cuda_stream
        self._args = (ctypes.byref(self._p), _ptr(q), _ptr(k_suf), _ptr(v_suf), _ptr(k_pre), _ptr(v_pre),
                      _ptr(suf_len), _ptr(out), _ptr(lse), None, 0, ctypes.c_void_p(stream))
        self._fn = load().pskv_attn_fwd

    def __call__(self):
        rc = self._fn(*self._args)
        if rc != PSKV_OK:
            _raise(rc)


def make_multi_params(base: pskv_attn_params, Np: int, kp_stride_n: int = 0) -> pskv_multi_params:
    p = pskv_multi_params()
    p.base = base
    p.Np = int(Np)
    p.reserved = 0
    p.kp_stride_n = int(kp_stride_n)
    return p


def pskv_attn_multi_validate(p: pskv_multi_params) -> int:
    return int(load().pskv_attn_multi_validate(ctypes.byref(p)))


def _multi_setup(q, k_suf, v_suf, k_pre, v_pre, pre_len, suf_len, out, lse, impl, scale):
    import torch
    if k_pre is None or k_pre.dim() != 4 or tuple(v_pre.shape) != tuple(k_pre.shape) or v_pre.stride() != k_pre.stride():
        raise ValueError("k_pre/v_pre must be [Np,P,Hkv,D] with shared strides")
    Np = k_pre.shape[0]
    if pre_len is not None and (pre_len.dtype != torch.int32 or tuple(pre_len.shape) != (Np,)
                                or not pre_len.is_contiguous() or pre_len.device != q.device):
        raise ValueError("pre_len must be a contiguous int32 [Np] tensor on the same device")
    # one instruction's prefix has the [P,Hkv,D] form the single-prefix checks know
    _check_inputs(q, k_suf, v_suf, k_pre[0], v_pre[0], suf_len, out, lse)
    base = _params_from_tensors(q, k_suf, k_pre[0], out, impl, scale)
    return make_multi_params(base, Np, _stride(k_pre, 0, "k_pre"))


def pskv_attn_fwd_multi(q, k_suf, v_suf, k_pre, v_pre, pre_len=None, suf_len=None, out=None, lse=None,
                        impl: str = "auto", scale: float = 0.0, stream: Optional[int] = None):
    """Batched multi-instruction forward call: k_pre, v_pre are [Np,P,Hkv,D] (left-padded,
    pre_len [Np] real rows each), candidate b belongs to instruction b // (B // Np)."""
    import torch
    if out is None:
        out = torch.empty_like(q)
    p = _multi_setup(q, k_suf, v_suf, k_pre, v_pre, pre_len, suf_len, out, lse, impl, scale)
    if stream is None:
        stream = torch.cuda.current_stream(q.device).cuda_stream
    with torch.cuda.device(q.device):
        rc = load().pskv_attn_fwd_multi(ctypes.byref(p), _ptr(q), _ptr(k_suf), _ptr(v_suf), _ptr(k_pre),
                                        _ptr(v_pre), _ptr(pre_len), _ptr(suf_len), _ptr(out), _ptr(lse),
                                        None, 0, ctypes.c_void_p(stream))
    if rc != PSKV_OK:
        _raise(rc)
    return out


class PreparedMultiCall:
    """pskv_attn_fwd_multi with every argument marshalled once (see PreparedCall)."""

    def __init__(self, q, k_suf, v_suf, k_pre, v_pre, pre_len, suf_len, out, lse=None, impl: str = "auto",
                 scale: float = 0.0, stream: Optional[int] = None):
        import torch
        self._keep = (q, k_suf, v_suf, k_pre, v_pre, pre_len, suf_len, out, lse)
        self._p = _multi_setup(q, k_suf, v_suf, k_pre, v_pre, pre_len, suf_len, out, lse, impl, scale)
        if stream is None:
            stream = torch.cuda.current_stream(q.device).cuda_stream
        self._args = (ctypes.byref(self._p), _ptr(q), _ptr(k_suf), _ptr(v_suf), _ptr(k_pre), _ptr(v_pre),
                      _ptr(pre_len), _ptr(suf_len), _ptr(out), _ptr(lse), None, 0, ctypes.c_void_p(stream))
        self._fn = load().pskv_attn_fwd_multi

    def __call__(self):
        rc = self._fn(*self._args)
        if rc != PSKV_OK:
            _raise(rc)


def _bwd_workspace(p, workspace, device, own_stream: bool):
    """The scratch tensor to hand to a backward call: the caller's, or a fresh one from torch
    (workspace=None), or none at all (workspace=False).  A fresh one goes back to torch's allocator
    when the call returns, which is only safe while the kernels run on torch's current stream (the
    allocator orders reuse by that stream): with a raw stream of the caller's the call does without
    scratch unless the caller brings a tensor and keeps it alive."""
    import torch
    if workspace is False or (workspace is None and own_stream):
        return None, 0
    if workspace is None:
        need = int(load().pskv_attn_bwd_workspace_bytes(ctypes.byref(p)))
        if need >= 1 << 62:      # invalid parameters: the call itself reports what is wrong
            return None, 0
        workspace = torch.empty(need, dtype=torch.uint8, device=device)
    return workspace, workspace.numel() * workspace.element_size()


def pskv_attn_bwd(q, k_suf, v_suf, k_pre, v_pre, suf_len, out, lse, dout, dq=None, dk_suf=None, dv_suf=None,
                  impl: str = "auto", scale: float = 0.0, stream: Optional[int] = None, workspace=None):
    """Enqueue the backward pass (gradients with respect to q, k_suf, v_suf; the prefix is a
    constant).  out and lse are the forward results; dout is laid out like out.  Gradient
    tensors are allocated by torch when not given (dq like q, dk_suf/dv_suf like k_suf), and so is
    the scratch tensor (workspace: a tensor to use instead, or False for a call without scratch).
    Returns (dq, dk_suf, dv_suf)."""
    import torch
    if lse is None:
        raise ValueError("the backward pass needs the forward pass's lse")
    _check_inputs(q, k_suf, v_suf, k_pre, v_pre, suf_len, out, lse)
    if tuple(dout.shape) != tuple(out.shape) or dout.stride() != out.stride() or dout.dtype != q.dtype:
        raise ValueError("dout must have the shape, strides and dtype of out")
    dq = torch.empty_like(q) if dq is None else dq
    dk_suf = torch.empty_like(k_suf) if dk_suf is None else dk_suf
    dv_suf = torch.empty_like(v_suf) if dv_suf is None else dv_suf
    if dq.shape != q.shape or dq.stride() != q.stride() or dq.dtype != q.dtype:
        raise ValueError("dq must have the shape, strides and dtype of q")
    for name, t in (("dk_suf", dk_suf), ("dv_suf", dv_suf)):
        if t.shape != k_suf.shape or t.stride() != k_suf.stride() or t.dtype != q.dtype:
            raise ValueError(f"{name} must have the shape, strides and dtype of k_suf")
    p = _params_from_tensors(q, k_suf, k_pre, out, impl, scale)
    ws, ws_bytes = _bwd_workspace(p, workspace, q.device, stream is not None)
    if stream is None:
        stream = torch.cuda.current_stream(q.device).cuda_stream
    with torch.cuda.device(q.device):
        rc = load().pskv_attn_bwd(ctypes.byref(p), _ptr(q), _ptr(k_suf), _ptr(v_suf), _ptr(k_pre), _ptr(v_pre),
                                  _ptr(suf_len), _ptr(out), _ptr(lse), _ptr(dout), _ptr(dq), _ptr(dk_suf),
                                  _ptr(dv_suf), _ptr(ws), ws_bytes, ctypes.c_void_p(stream))
    if rc != PSKV_OK:
        _raise(rc)
    return dq, dk_suf, dv_suf


def pskv_attn_bwd_multi(q, k_suf, v_suf, k_pre, v_pre, pre_len, suf_len, out, lse, dout, dq=None, dk_suf=None,
                        dv_suf=None, impl: str = "auto", scale: float = 0.0, stream: Optional[int] = None,
                        workspace=None):
    """Backward pass of the batched multi-instruction form (arguments as for pskv_attn_fwd_multi
    and pskv_attn_bwd).  Returns (dq, dk_suf, dv_suf)."""
    import torch
    if lse is None:
        raise ValueError("the backward pass needs the forward pass's lse")
    p = _multi_setup(q, k_suf, v_suf, k_pre, v_pre, pre_len, suf_len, out, lse, impl, scale)
    if tuple(dout.shape) != tuple(out.shape) or dout.stride() != out.stride() or dout.dtype != q.dtype:
        raise ValueError("dout must have the shape, strides and dtype of out")
    dq = torch.empty_like(q) if dq is None else dq
    dk_suf = torch.empty_like(k_suf) if dk_suf is None else dk_suf
    dv_suf = torch.empty_like(v_suf) if dv_suf is None else dv_suf
    if dq.shape != q.shape or dq.stride() != q.stride() or dq.dtype != q.dtype:
        raise ValueError("dq must have the shape, strides and dtype of q")
    for name, t in (("dk_suf", dk_suf), ("dv_suf", dv_suf)):
        if t.shape != k_suf.shape or t.stride() != k_suf.stride() or t.dtype != q.dtype:
            raise ValueError(f"{name} must have the shape, strides and dtype of k_suf")
    ws, ws_bytes = _bwd_workspace(p.base, workspace, q.device, stream is not None)
    if stream is None:
        stream = torch.cuda.current_stream(q.device).cuda_stream
    with torch.cuda.device(q.device):
        rc = load().pskv_attn_bwd_multi(ctypes.byref(p), _ptr(q), _ptr(k_suf), _ptr(v_suf), _ptr(k_pre), _ptr(v_pre),
                                        _ptr(pre_len), _ptr(suf_len), _ptr(out), _ptr(lse), _ptr(dout), _ptr(dq),
                                        _ptr(dk_suf), _ptr(dv_suf), _ptr(ws), ws_bytes, ctypes.c_void_p(stream))
    if rc != PSKV_OK:
        _raise(rc)
    return dq, dk_suf, dv_suf


def pskv_attn_bwd_noalloc(q, k_suf, v_suf, k_pre, v_pre, suf_len, out, lse, dout, dq, dk_suf, dv_suf,
                          impl: str = "auto", scale: float = 0.0, stream: Optional[int] = None):
    """pskv_attn_bwd through the entry point that allocates nothing: the gradient tensors are the
    caller's, the scratch is the library's built-in array (refused with PSKV_ERR_WORKSPACE when
    B*Hq*S*4 exceeds PSKV_NOALLOC_SCRATCH_BYTES), and this wrapper creates no tensor either."""
    import torch
    if lse is None:
        raise ValueError("the backward pass needs the forward pass's lse")
    _check_inputs(q, k_suf, v_suf, k_pre, v_pre, suf_len, out, lse)
    if tuple(dout.shape) != tuple(out.shape) or dout.stride() != out.stride() or dout.dtype != q.dtype:
        raise ValueError("dout must have the shape, strides and dtype of out")
    if dq.shape != q.shape or dq.stride() != q.stride() or dq.dtype != q.dtype:
        raise ValueError("dq must have the shape, strides and dtype of q")
    for name, t in (("dk_suf", dk_suf), ("dv_suf", dv_suf)):
        if t.shape != k_suf.shape or t.stride() != k_suf.stride() or t.dtype != q.dtype:
            raise ValueError(f"{name} must have the shape, strides and dtype of k_suf")
    p = _params_from_tensors(q, k_suf, k_pre, out, impl, scale)
    if stream is None:
        stream = torch.cuda.current_stream(q.device).cuda_stream
    with torch.cuda.device(q.device):
        rc = load().pskv_attn_bwd_noalloc(ctypes.byref(p), _ptr(q), _ptr(k_suf), _ptr(v_suf), _ptr(k_pre), _ptr(v_pre),
                                          _ptr(suf_len), _ptr(out), _ptr(lse), _ptr(dout), _ptr(dq), _ptr(dk_suf),
                                          _ptr(dv_suf), ctypes.c_void_p(stream))
    if rc != PSKV_OK:
        _raise(rc)
    return dq, dk_suf, dv_suf
