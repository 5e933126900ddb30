"""Seeded synthetic workloads for batched candidate-suffix attention.

This module produces *data only*: tensor shapes, lengths and N(0,1) values with the
shapes of the paper's workloads (prompt of roughly 80-250 tokens as the shared prefix,
suffix-side segments of 20-160 tokens, MHA 32/32, GQA 32/8 and 28/4 head layouts, head
dimension 128; Table 1 and Table 8 of the paper).  It contains none of the method's
arithmetic, so both the CPU oracle's tests and the HIP path's tests may draw from it.

bf16 tensors are carried on the host as ``uint16`` bit patterns (NumPy has no bf16);
the same bits go to the oracle and to the GPU.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np

BASE_SEED = 20260313


@dataclass(frozen=True)
class Workload:
    """One attention-layer problem: B candidates, shared prefix P, padded suffix S."""
    name: str
    B: int
    P: int
    S: int
    len_lo: int          # suffix lengths drawn uniformly in [len_lo, len_hi]
    len_hi: int
    Hq: int
    Hkv: int
    D: int
    dtype: str           # "f32" or "bf16"
    index: int           # position in the list of named workloads (seed offset)

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index


WORKLOADS: Dict[str, Workload] = {w.name: w for w in [
    Workload("tiny_f32",       8,    48,   16,  8, 16,  4,  4,  64, "f32",  0),
    Workload("mha7b_bf16",     512,  128,  20, 20, 20, 32, 32, 128, "bf16", 1),
    Workload("gqa8b_bf16",     1024, 256,  24, 16, 24, 32,  8, 128, "bf16", 2),
    Workload("longprefix_bf16", 256, 2048, 32, 32, 32, 32,  8, 128, "bf16", 3),
    Workload("mha13b_bf16",    4096, 512,  64, 32, 64, 40, 40, 128, "bf16", 4),
    # The scoring workload with the chat template's tail and the target appended to the
    # suffix (Sec. 3.1: the decoded segment is suffix + target): about 20 + 93 + a few dozen
    # tokens after a prompt of about 80-130, on the 32/8 and the 28/4 (group of 7, Table 8)
    # head layouts.
    Workload("ldec_gqa8b_bf16", 256, 128, 160, 128, 160, 32, 8, 128, "bf16", 5),
    Workload("ldec_qwen7b_bf16", 256, 128, 160, 128, 160, 28, 4, 128, "bf16", 6),
]}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even), returned as uint16 bits.
    NaN stays NaN (quiet)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    out = rounded.astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out = np.where(nan, np.uint16(0x7FC0), out).astype(np.uint16)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Inputs:
    """Host-side tensors of one problem. For dtype "bf16" the q/k/v arrays are uint16 bits."""
    w: Workload
    q: np.ndarray        # [B,S,Hq,D]
    k_suf: np.ndarray    # [B,S,Hkv,D]
    v_suf: np.ndarray    # [B,S,Hkv,D]
    k_pre: np.ndarray    # [P,Hkv,D]
    v_pre: np.ndarray    # [P,Hkv,D]
    suf_len: np.ndarray  # [B] int32
    scale: float
    meta: dict = field(default_factory=dict)

    def as_f32(self, name: str) -> np.ndarray:
        a = getattr(self, name)
        return bf16_bits_to_f32(a) if self.w.dtype == "bf16" else a

    def take(self, cand: np.ndarray) -> "Inputs":
        """The same problem restricted to the listed candidates (prefix unchanged)."""
        cand = np.asarray(cand, dtype=np.int64)
        w = Workload(self.w.name + "_subset", len(cand), self.w.P, self.w.S, self.w.len_lo,
                     self.w.len_hi, self.w.Hq, self.w.Hkv, self.w.D, self.w.dtype, self.w.index)
        return Inputs(w, np.ascontiguousarray(self.q[cand]),
                      np.ascontiguousarray(self.k_suf[cand]),
                      np.ascontiguousarray(self.v_suf[cand]),
                      self.k_pre, self.v_pre,
                      np.ascontiguousarray(self.suf_len[cand]), self.scale,
                      dict(self.meta, subset=cand))


CAND_BLOCK = 64   # candidates per independent random stream (fixed: part of the recipe)


def make_inputs(w: Workload, pad: str = "nan", seed: Optional[int] = None,
                workers: int = 8) -> Inputs:
    """Draw one problem, deterministically from the workload's seed.

    Streams (children of ``SeedSequence(seed)``): child 0 draws suf_len (uniform integers,
    inclusive), child 1 draws k_pre then v_pre, child 2+n draws q, k_suf, v_suf of the n-th
    block of 64 candidates.  All values are float32 N(0,1) draws; bf16 workloads round them
    to bf16 (RNE).  Blocks are independent, so they are drawn by a small thread pool.

    pad = "nan": rows at or beyond a candidate's length are filled with NaN (tests:
                 a padded row must never reach a valid output);
    pad = "zero": filled with 0 (benchmarks);
    pad = "keep": left as the N(0,1) draws.
    """
    from concurrent.futures import ThreadPoolExecutor

    nblk = (w.B + CAND_BLOCK - 1) // CAND_BLOCK
    children = np.random.SeedSequence(w.seed if seed is None else seed).spawn(2 + nblk)
    suf_len = np.random.default_rng(children[0]).integers(
        w.len_lo, w.len_hi + 1, size=w.B, dtype=np.int64).astype(np.int32)
    bf16 = w.dtype == "bf16"
    store = np.uint16 if bf16 else np.float32
    fill = {"nan": np.float32(np.nan), "zero": np.float32(0.0)}.get(pad)

    def finish(a):
        return f32_to_bf16_bits(a) if bf16 else a

    rng_p = np.random.default_rng(children[1])
    k_pre = finish(rng_p.standard_normal(size=(w.P, w.Hkv, w.D), dtype=np.float32))
    v_pre = finish(rng_p.standard_normal(size=(w.P, w.Hkv, w.D), dtype=np.float32))

    q = np.empty((w.B, w.S, w.Hq, w.D), dtype=store)
    k_suf = np.empty((w.B, w.S, w.Hkv, w.D), dtype=store)
    v_suf = np.empty((w.B, w.S, w.Hkv, w.D), dtype=store)

    def block(n):
        lo, hi = n * CAND_BLOCK, min(w.B, (n + 1) * CAND_BLOCK)
        rng = np.random.default_rng(children[2 + n])
        padded = np.arange(w.S)[None, :] >= suf_len[lo:hi, None]
        for dst, heads in ((q, w.Hq), (k_suf, w.Hkv), (v_suf, w.Hkv)):
            a = rng.standard_normal(size=(hi - lo, w.S, heads, w.D), dtype=np.float32)
            if fill is not None:
                a[padded] = fill
            dst[lo:hi] = finish(a)

    with ThreadPoolExecutor(max_workers=max(1, workers)) as ex:
        list(ex.map(block, range(nblk)))
    # the softmax scale 1/sqrt(D) as the fp32 number the C ABI carries; the same value goes to both sides
    scale = float(np.float32(1.0 / np.sqrt(w.D)))
    return Inputs(w, q, k_suf, v_suf, k_pre, v_pre, suf_len, scale, {"pad": pad})


def custom_workload(name, B, P, S, len_lo, len_hi, Hq, Hkv, D, dtype, index=100) -> Workload:
    return Workload(name, B, P, S, len_lo, len_hi, Hq, Hkv, D, dtype, index)


# ---------------------------------------------------------------------------------------------
# Batched multi-instruction form (Sec. 4.3 of the paper): Np instructions with their own
# left-padded prefixes and C candidates each.
# ---------------------------------------------------------------------------------------------
@dataclass(frozen=True)
class MultiWorkload:
    name: str
    Np: int              # instructions
    C: int               # candidates per instruction (B = Np * C)
    P: int               # padded prefix length
    pre_lo: int          # real prefix lengths drawn uniformly in [pre_lo, pre_hi]
    pre_hi: int
    S: int
    len_lo: int
    len_hi: int
    Hq: int
    Hkv: int
    D: int
    dtype: str
    index: int

    @property
    def B(self) -> int:
        return self.Np * self.C

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def seed(self) -> int:
        return BASE_SEED + 1000 + self.index


MULTI_WORKLOADS: Dict[str, MultiWorkload] = {w.name: w for w in [
    # 8 instructions of 78-250 prompt tokens (Sec. 3: prompts of roughly 80 tokens plus the chat
    # template), 128 candidates each, the 8B-class GQA head layout
    MultiWorkload("multi8_gqa8b_bf16",  8, 128, 256,  96, 256, 24, 16, 24, 32, 8, 128, "bf16", 0),
    # 32 instructions, 32 candidates each (more virtual heads than one pass of workgroups)
    MultiWorkload("multi32_gqa8b_bf16", 32, 32, 256,  96, 256, 24, 16, 24, 32, 8, 128, "bf16", 1),
    # long, unevenly padded prefixes streamed through LDS
    MultiWorkload("multi4_long_bf16",   4,  64, 1024, 300, 1024, 32, 32, 32, 32, 8, 128, "bf16", 2),
]}


@dataclass
class MultiInputs:
    w: MultiWorkload
    q: np.ndarray        # [B,S,Hq,D]
    k_suf: np.ndarray    # [B,S,Hkv,D]
    v_suf: np.ndarray
    k_pre: np.ndarray    # [Np,P,Hkv,D], left-padded
    v_pre: np.ndarray
    pre_len: np.ndarray  # [Np] int32
    suf_len: np.ndarray  # [B] int32
    scale: float
    meta: dict = field(default_factory=dict)

    def take_instructions(self, which: np.ndarray) -> "MultiInputs":
        """The same problem restricted to the listed instructions and all their candidates."""
        which = np.asarray(which, dtype=np.int64)
        cand = (which[:, None] * self.w.C + np.arange(self.w.C)[None, :]).reshape(-1)
        w = MultiWorkload(self.w.name + "_subset", len(which), self.w.C, self.w.P, self.w.pre_lo, self.w.pre_hi,
                          self.w.S, self.w.len_lo, self.w.len_hi, self.w.Hq, self.w.Hkv, self.w.D, self.w.dtype,
                          self.w.index)
        c = np.ascontiguousarray
        return MultiInputs(w, c(self.q[cand]), c(self.k_suf[cand]), c(self.v_suf[cand]), c(self.k_pre[which]),
                           c(self.v_pre[which]), c(self.pre_len[which]), c(self.suf_len[cand]), self.scale,
                           dict(self.meta, instructions=which))


def make_multi_inputs(w: MultiWorkload, pad: str = "nan", seed: Optional[int] = None) -> MultiInputs:
    """Draw one multi-instruction problem.  Streams (children of ``SeedSequence(seed)``): child 0
    draws pre_len then suf_len (uniform integers, inclusive), child 1 draws k_pre then v_pre,
    child 2+n draws q, k_suf, v_suf of the n-th block of 64 candidates.  N(0,1) float32 draws,
    rounded to bf16 (RNE) for bf16 workloads.  Prefix rows before an instruction's real rows
    and suffix rows at or beyond a candidate's length are padding: NaN for pad="nan", 0 for
    pad="zero", the draws themselves for pad="keep"."""
    nblk = (w.B + CAND_BLOCK - 1) // CAND_BLOCK
    children = np.random.SeedSequence(w.seed if seed is None else seed).spawn(2 + nblk)
    rng0 = np.random.default_rng(children[0])
    pre_len = rng0.integers(w.pre_lo, w.pre_hi + 1, size=w.Np, dtype=np.int64).astype(np.int32)
    suf_len = rng0.integers(w.len_lo, w.len_hi + 1, size=w.B, dtype=np.int64).astype(np.int32)
    bf16 = w.dtype == "bf16"
    store = np.uint16 if bf16 else np.float32
    fill = {"nan": np.float32(np.nan), "zero": np.float32(0.0)}.get(pad)

    def finish(a):
        return f32_to_bf16_bits(a) if bf16 else a

    rng_p = np.random.default_rng(children[1])
    pre_pad = np.arange(w.P)[None, :] < (w.P - pre_len)[:, None]     # [Np,P]: True on left padding
    pre = []
    for _ in range(2):
        a = rng_p.standard_normal(size=(w.Np, w.P, w.Hkv, w.D), dtype=np.float32)
        if fill is not None:
            a[pre_pad] = fill
        pre.append(finish(a))
    q = np.empty((w.B, w.S, w.Hq, w.D), dtype=store)
    k_suf = np.empty((w.B, w.S, w.Hkv, w.D), dtype=store)
    v_suf = np.empty((w.B, w.S, w.Hkv, w.D), dtype=store)
    for n in range(nblk):
        lo, hi = n * CAND_BLOCK, min(w.B, (n + 1) * CAND_BLOCK)
        rng = np.random.default_rng(children[2 + n])
        padded = np.arange(w.S)[None, :] >= suf_len[lo:hi, None]
        for dst, heads in ((q, w.Hq), (k_suf, w.Hkv), (v_suf, w.Hkv)):
            a = rng.standard_normal(size=(hi - lo, w.S, heads, w.D), dtype=np.float32)
            if fill is not None:
                a[padded] = fill
            dst[lo:hi] = finish(a)
    scale = float(np.float32(1.0 / np.sqrt(w.D)))
    return MultiInputs(w, q, k_suf, v_suf, pre[0], pre[1], pre_len, suf_len, scale, {"pad": pad})


def custom_multi_workload(name, Np, C, P, pre_lo, pre_hi, S, len_lo, len_hi, Hq, Hkv, D, dtype, index=100):
    return MultiWorkload(name, Np, C, P, pre_lo, pre_hi, S, len_lo, len_hi, Hq, Hkv, D, dtype, index)


# ---------------------------------------------------------------------------------------------
# Host tensors <-> torch tensors on the GPU (data movement only), and the seeded incoming gradient
# of the backward pass.
# ---------------------------------------------------------------------------------------------
def _to_torch(a: np.ndarray, dtype: str, device):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype == "bf16":
        t = t.view(torch.bfloat16)
    return t.to(device)


def to_device(inp: Inputs, device="cuda:0") -> dict:
    """The problem's tensors on the GPU, keyed like the arguments of pskv_attn_fwd (k_pre, v_pre None when P == 0)."""
    import torch
    dt = inp.w.dtype
    return dict(q=_to_torch(inp.q, dt, device), k_suf=_to_torch(inp.k_suf, dt, device), v_suf=_to_torch(inp.v_suf, dt, device),
                k_pre=_to_torch(inp.k_pre, dt, device) if inp.w.P > 0 else None,
                v_pre=_to_torch(inp.v_pre, dt, device) if inp.w.P > 0 else None,
                suf_len=torch.from_numpy(inp.suf_len).to(device))


def to_device_multi(inp: MultiInputs, device="cuda:0") -> dict:
    import torch
    dt = inp.w.dtype
    return dict(q=_to_torch(inp.q, dt, device), k_suf=_to_torch(inp.k_suf, dt, device), v_suf=_to_torch(inp.v_suf, dt, device),
                k_pre=_to_torch(inp.k_pre, dt, device), v_pre=_to_torch(inp.v_pre, dt, device),
                pre_len=torch.from_numpy(inp.pre_len).to(device), suf_len=torch.from_numpy(inp.suf_len).to(device))


def out_to_f64(t) -> np.ndarray:
    """A result tensor of the GPU as float64 on the host (bf16 widened exactly)."""
    import torch
    if t.dtype == torch.bfloat16:
        return bf16_bits_to_f32(t.view(torch.uint16).cpu().numpy()).astype(np.float64)
    return t.cpu().numpy().astype(np.float64)


def make_dout(inp, seed: int):
    """Seeded N(0,1) incoming gradient of the backward pass in the workload's storage type, NaN on
    padded rows.  Returns (host array in storage form, the same values as float64)."""
    w = inp.w
    rng = np.random.default_rng(seed)
    a = rng.standard_normal(size=(w.B, w.S, w.Hq, w.D), dtype=np.float32)
    a[np.arange(w.S)[None, :] >= inp.suf_len[:, None]] = np.nan
    if w.dtype == "bf16":
        bits = f32_to_bf16_bits(a)
        return bits, bf16_bits_to_f32(bits).astype(np.float64)
    return a, a.astype(np.float64)
