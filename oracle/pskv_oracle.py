"""Python face of the CPU oracle (TEST INFRASTRUCTURE ONLY, never on the product path).

Two independent-of-the-GPU implementations of the same definition (paper Eq. 2 with the
Standard-KV prefix repetition of Eq. 3):

* ``attn``        calls the plain C program ``pskv_oracle.c`` (double precision, OpenMP over
                  (candidate, KV head)); used for parity at realistic sizes and for the
                  benchmark's cpu_baseline timing;
* ``attn_numpy``  the same steps spelled with NumPy float64 ops, for small cases and as a
                  second opinion on the C program.

bf16 inputs are ``uint16`` bit patterns and are widened exactly.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pskv_oracle.c")
_LIB = os.path.join(_HERE, "libpskv_oracle.so")
_DT = {"f32": 0, "bf16": 1, "f64": 2}
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-fno-fast-math",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.pskv_oracle_attn.restype = ctypes.c_int
        lib.pskv_oracle_attn.argtypes = [ctypes.c_int] * 7 + [ctypes.c_double] + \
            [ctypes.c_void_p] * 9 + [ctypes.c_int]
        lib.pskv_oracle_attn_multi.restype = ctypes.c_int
        lib.pskv_oracle_attn_multi.argtypes = [ctypes.c_int] * 8 + [ctypes.c_double] + \
            [ctypes.c_void_p] * 10 + [ctypes.c_int]
        lib.pskv_oracle_attn_bwd.restype = ctypes.c_int
        lib.pskv_oracle_attn_bwd.argtypes = [ctypes.c_int] * 7 + [ctypes.c_double] + \
            [ctypes.c_void_p] * 10 + [ctypes.c_int]
        lib.pskv_oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def threads() -> int:
    return int(_load().pskv_oracle_threads())


def _check(a: np.ndarray, shape, dtype: str, name: str) -> np.ndarray:
    want = {"f32": np.float32, "bf16": np.uint16, "f64": np.float64}[dtype]
    if a.dtype != want:
        raise TypeError(f"{name}: dtype {a.dtype}, expected {want}")
    if tuple(a.shape) != tuple(shape):
        raise ValueError(f"{name}: shape {a.shape}, expected {shape}")
    return np.ascontiguousarray(a)


def attn(q, k_suf, v_suf, k_pre, v_pre, suf_len, scale: float, dtype: str,
         want_lse: bool = False, want_probs: bool = False, nthreads: int = 0):
    """Run the C oracle. Returns out [B,S,Hq,D] float64 (+ lse [B,Hq,S], + probs [B,Hq,S,P+S])."""
    B, S, Hq, D = q.shape
    Hkv = k_suf.shape[2]
    P = k_pre.shape[0]
    q = _check(q, (B, S, Hq, D), dtype, "q")
    k_suf = _check(k_suf, (B, S, Hkv, D), dtype, "k_suf")
    v_suf = _check(v_suf, (B, S, Hkv, D), dtype, "v_suf")
    k_pre = _check(k_pre, (P, Hkv, D), dtype, "k_pre")
    v_pre = _check(v_pre, (P, Hkv, D), dtype, "v_pre")
    sl = None
    if suf_len is not None:
        sl = np.ascontiguousarray(suf_len, dtype=np.int32)
        if sl.shape != (B,):
            raise ValueError("suf_len shape")
    out = np.empty((B, S, Hq, D), dtype=np.float64)
    lse = np.empty((B, Hq, S), dtype=np.float64) if want_lse else None
    probs = np.empty((B, Hq, S, P + S), dtype=np.float64) if want_probs else None

    def ptr(a):
        return None if a is None else a.ctypes.data_as(ctypes.c_void_p)

    rc = _load().pskv_oracle_attn(B, S, P, Hq, Hkv, D, _DT[dtype], float(scale),
                                  ptr(q), ptr(k_suf), ptr(v_suf), ptr(k_pre), ptr(v_pre),
                                  ptr(sl), ptr(out), ptr(lse), ptr(probs), int(nthreads))
    if rc != 0:
        raise RuntimeError(f"pskv_oracle_attn failed with code {rc}")
    res = (out,)
    if want_lse:
        res += (lse,)
    if want_probs:
        res += (probs,)
    return res[0] if len(res) == 1 else res


def attn_bwd(q, k_suf, v_suf, k_pre, v_pre, suf_len, dout, scale: float, dtype: str, nthreads: int = 0):
    """Gradient of sum(dout * attn(...)) with respect to q, k_suf, v_suf (prefix constant).
    dout is float64 [B,S,Hq,D].  Returns (dq, dk_suf, dv_suf), float64."""
    B, S, Hq, D = q.shape
    Hkv = k_suf.shape[2]
    P = k_pre.shape[0]
    q = _check(q, (B, S, Hq, D), dtype, "q")
    k_suf = _check(k_suf, (B, S, Hkv, D), dtype, "k_suf")
    v_suf = _check(v_suf, (B, S, Hkv, D), dtype, "v_suf")
    k_pre = _check(k_pre, (P, Hkv, D), dtype, "k_pre")
    v_pre = _check(v_pre, (P, Hkv, D), dtype, "v_pre")
    dout = _check(dout, (B, S, Hq, D), "f64", "dout")
    sl = None if suf_len is None else np.ascontiguousarray(suf_len, dtype=np.int32)
    dq = np.empty((B, S, Hq, D), dtype=np.float64)
    dk = np.empty((B, S, Hkv, D), dtype=np.float64)
    dv = np.empty((B, S, Hkv, D), dtype=np.float64)

    def ptr(a):
        return None if a is None else a.ctypes.data_as(ctypes.c_void_p)

    rc = _load().pskv_oracle_attn_bwd(B, S, P, Hq, Hkv, D, _DT[dtype], float(scale),
                                      ptr(q), ptr(k_suf), ptr(v_suf), ptr(k_pre), ptr(v_pre), ptr(sl),
                                      ptr(dout), ptr(dq), ptr(dk), ptr(dv), int(nthreads))
    if rc != 0:
        raise RuntimeError(f"pskv_oracle_attn_bwd failed with code {rc}")
    return dq, dk, dv


def attn_bwd_multi(q, k_suf, v_suf, k_pre, v_pre, pre_len, suf_len, dout, scale: float, dtype: str,
                   nthreads: int = 0):
    """Backward pass of the batched multi-instruction form (Sec. 4.3).  The instructions are
    independent problems: instruction n is the single-prefix problem made of its own C = B / Np
    candidates and of the real rows of its prefix, the last pre_len[n] of the Pp padded ones
    (App. F.1: prefixes are left-padded), so its gradient is attn_bwd of exactly that problem.
    Returns (dq, dk_suf, dv_suf), float64."""
    B = q.shape[0]
    Np, Pp = k_pre.shape[0], k_pre.shape[1]
    if Np == 0 or B % Np != 0:
        raise ValueError("the number of candidates must be a multiple of the number of instructions")
    C = B // Np
    dq = np.empty(q.shape, dtype=np.float64)
    dk = np.empty(k_suf.shape, dtype=np.float64)
    dv = np.empty(v_suf.shape, dtype=np.float64)
    for n in range(Np):
        pl = Pp if pre_len is None else min(max(int(pre_len[n]), 0), Pp)
        cs = slice(n * C, (n + 1) * C)
        sl = None if suf_len is None else np.asarray(suf_len)[cs]
        dq[cs], dk[cs], dv[cs] = attn_bwd(q[cs], k_suf[cs], v_suf[cs], k_pre[n, Pp - pl:], v_pre[n, Pp - pl:], sl,
                                          np.asarray(dout)[cs], scale, dtype, nthreads)
    return dq, dk, dv


def attn_multi(q, k_suf, v_suf, k_pre, v_pre, pre_len, suf_len, scale: float, dtype: str,
               want_lse: bool = False, want_probs: bool = False, nthreads: int = 0):
    """Batched multi-instruction form (Sec. 4.3): k_pre, v_pre are [Np,Pp,Hkv,D], left-padded,
    with pre_len [Np] real rows each; candidate b belongs to instruction b // (B // Np).
    Returns out [B,S,Hq,D] float64 (+ lse [B,Hq,S], + probs [B,Hq,S,Pp+S])."""
    B, S, Hq, D = q.shape
    Hkv = k_suf.shape[2]
    Np, Pp = k_pre.shape[0], k_pre.shape[1]
    if Np == 0 or B % Np != 0:
        raise ValueError("the number of candidates must be a multiple of the number of instructions")
    C = B // Np
    q = _check(q, (B, S, Hq, D), dtype, "q")
    k_suf = _check(k_suf, (B, S, Hkv, D), dtype, "k_suf")
    v_suf = _check(v_suf, (B, S, Hkv, D), dtype, "v_suf")
    k_pre = _check(k_pre, (Np, Pp, Hkv, D), dtype, "k_pre")
    v_pre = _check(v_pre, (Np, Pp, Hkv, D), dtype, "v_pre")
    pl = None if pre_len is None else np.ascontiguousarray(pre_len, dtype=np.int32)
    sl = None if suf_len is None else np.ascontiguousarray(suf_len, dtype=np.int32)
    if pl is not None and pl.shape != (Np,):
        raise ValueError("pre_len shape")
    if sl is not None and sl.shape != (B,):
        raise ValueError("suf_len shape")
    out = np.empty((B, S, Hq, D), dtype=np.float64)
    lse = np.empty((B, Hq, S), dtype=np.float64) if want_lse else None
    probs = np.empty((B, Hq, S, Pp + S), dtype=np.float64) if want_probs else None

    def ptr(a):
        return None if a is None else a.ctypes.data_as(ctypes.c_void_p)

    rc = _load().pskv_oracle_attn_multi(Np, C, S, Pp, Hq, Hkv, D, _DT[dtype], float(scale),
                                        ptr(q), ptr(k_suf), ptr(v_suf), ptr(k_pre), ptr(v_pre),
                                        ptr(pl), ptr(sl), ptr(out), ptr(lse), ptr(probs), int(nthreads))
    if rc != 0:
        raise RuntimeError(f"pskv_oracle_attn_multi failed with code {rc}")
    res = (out,)
    if want_lse:
        res += (lse,)
    if want_probs:
        res += (probs,)
    return res[0] if len(res) == 1 else res


def _widen(a: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def attn_numpy(q, k_suf, v_suf, k_pre, v_pre, suf_len, scale: float, dtype: str
               ) -> Tuple[np.ndarray, np.ndarray]:
    """NumPy float64 spelling of the same definition. Returns (out, lse)."""
    q, k_suf, v_suf, k_pre, v_pre = (_widen(a, dtype) for a in (q, k_suf, v_suf, k_pre, v_pre))
    B, S, Hq, D = q.shape
    Hkv = k_suf.shape[2]
    P = k_pre.shape[0]
    G = Hq // Hkv
    out = np.zeros((B, S, Hq, D))
    lse = np.full((B, Hq, S), -np.inf)
    for b in range(B):
        n = S if suf_len is None else int(suf_len[b])
        if n == 0:
            continue
        for h in range(Hq):
            k = h // G
            # Eq. 3: a private copy of the prefix for this candidate, suffix rows appended
            Kfull = np.concatenate([k_pre[:, k, :].copy(), k_suf[b, :n, k, :]], axis=0)
            Vfull = np.concatenate([v_pre[:, k, :].copy(), v_suf[b, :n, k, :]], axis=0)
            s = (q[b, :n, h, :] @ Kfull.T) * scale                       # [n, P+n]
            col = np.arange(P + n)[None, :]
            row = np.arange(n)[:, None]
            s = np.where(col <= P + row, s, -np.inf)                      # prefix + causal
            m = s.max(axis=1, keepdims=True)
            e = np.exp(s - m)
            den = e.sum(axis=1, keepdims=True)
            out[b, :n, h, :] = (e / den) @ Vfull                           # Eq. 2
            lse[b, h, :n] = (m + np.log(den))[:, 0]
    return out, lse


def alg_flops(suf_len: np.ndarray, P: int, Hq: int, D: int) -> int:
    """Multiply-add work over visible keys only, QK^T and PV at 2 FLOP per MAC
    (the L_dec(2 N_p + L_dec) count of App. B.1, with the diagonal included)."""
    l = np.asarray(suf_len, dtype=np.int64)
    return int((Hq * 4 * D * (l * P + l * (l + 1) // 2)).sum())
