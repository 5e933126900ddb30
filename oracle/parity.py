"""Comparison of a result with the CPU oracle under bounds derived from the kernels' arithmetic
(TEST INFRASTRUCTURE like the rest of this folder: used by tests/, by smoke() and by the self-check
of bench.py; never on the product path).  Problems are taken as objects with the fields of the
seeded input module (q, k_suf, v_suf, k_pre, v_pre, suf_len, scale, w); nothing of the HIP
package is imported here.

THE BARS (nothing below is fitted to a measurement; tests/test_tolerance_model.py checks the
derivation itself on the CPU by emulating the kernels' roundings on the oracle's exact
weights, and plants errors that must be caught).

Notation: u = 2^-8 is the unit round-off of bf16 (8 significant bits, round to nearest even:
|fl(x) - x| <= u |x|); eta collects every fp32 effect of the path (score accumulation, exp2,
the row sum of n terms, the fp32 accumulators, the reciprocal): eta = n 2^-23 + 2^-16 with n the
number of keys a row sees (twice the worst case n 2^-24 of an n-term fp32 sum, plus two units
of fp32 for the 128-term dot products and the exponential) - 5e-5 at n = 280, 1 % of u.

fp32 tensors, forward: every valid element within 1e-5 relative (the stated bar).

bf16 tensors, forward.  The exact result of Eq. 2 is out_d = sum_j w_j V_jd with softmax
weights w_j = e_j / L.  The matrix-core kernels round each unnormalised weight e_j to bf16
before the value product (relative error at most u, independent from key to key), form the
denominator L from the UNROUNDED weights in fp32, and round the quotient to bf16 once.  Hence

    |gpu_d - out_d|  <=  (u + eta) * A_d  +  u * |out_d|,     A_d = sum_j w_j |V_jd|,

a worst-case bound that holds element by element.  A is what the oracle returns when it is
handed |V| in place of V (the weights do not depend on V), so the bound costs one more oracle
call and no arithmetic of its own.  Three things are asserted:
  (1) the element-wise bound above, on every valid element;
  (2) max |gpu - ref| <= 2e-2, the stated bar taken literally;
  (3) rms(gpu - ref) <= sqrt(2/3) u * rms(ref) + eta * rms(A): the two roundings are
      independent with mean square at most u^2/3 of the rounded value each (a uniform error
      inside half a unit in the last place, worst position inside the binade), and the mean
      over V of (sum_j w_j eps_j V_jd)^2 is eps^2 sum_j w_j^2 = eps^2 E[out_d^2].  With
      mantissas spread log-uniformly the expected figure is 0.60 of that bar, 2.35e-3 rms(ref);
      a kernel that loses more than its roundings explain fails here long before (1).
The normalised figure max|err| / std(ref) is printed too but cannot be a bar at 2e-2 for any
bf16 result: the final rounding alone is up to u |out_d|, which exceeds 2e-2 std(ref) for every
element beyond 5.1 standard deviations, and 1e8 outputs reach 6.

Gradients (bf16).  The kernels form p_j = exp2(c s_j - lse) in fp32 from the forward pass's lse,
dp_j = <dout, V_j> on the matrix cores in fp32, delta~ = <dout, out> in fp32 from the forward
RESULT AS STORED (bf16), ds_j = p_j (dp_j - delta~); ds (for dq, dk) and p (for dv) are rounded to
bf16 before the second products and each gradient is rounded to bf16 once.  Element by element,

    |dq~ - dq|_d  <= scale [ (u + 2 eta) sum_j |ds_j| |K_jd|  +  (1 + u) sum_j p_j (E + C_j) |K_jd| ] + u |dq_d|
    |dk~ - dk|_jd <= scale sum_rows [ (u + 2 eta) |ds_rj| |q_rd|  +  (1 + u) p_rj (E_r + C_rj) |q_rd| ] + u |dk_jd|
    |dv~ - dv|_jd <= (u + 2 eta) sum_rows p_rj |dout_rd|  +  u |dv_jd|

with the sums over what the exact gradient sums over (grad_bounds() below spells them with
NumPy in float64; they are bounds, not expected values; 2 eta because p inherits the error of
lse as well).  C_j = eta sum_d |dout_d| (|V_jd| + |out_d|) is the fp32 noise of the two 128-term
dot products dp_j and delta~ where they cancel: a row that sees a single key has dp = delta
exactly and a vanishing gradient, and the kernels leave that noise there.  E bounds
|delta~ - delta|, the one place where the worst case is hopeless (it would let all 128 + n
rounding errors of the stored forward result line up with the signs of dout).  By the forward
model delta~ - delta = sum_j w_j eps_j dp_j + sum_d eps'_d dout_d out_d, a sum of independent
terms with |eps| <= u, so by Hoeffding's inequality

    |delta~ - delta| <= E = LAMBDA u sqrt( sum_j w_j^2 dp_j^2 + sum_d dout_d^2 out_d^2 ),   LAMBDA = 9,

fails with probability at most 2 exp(-LAMBDA^2 / 2) = 5e-18 per row.  No row is treated
differently from any other.  The rms error of each gradient is asserted as well:
sqrt(2/3) u rms(ref) for its two roundings as in (3), plus the rms of the delta term at its
expected size (the E part of the bound divided by sqrt(3) LAMBDA), plus the fp32 shares.
fp32 tensors: the same formulas with u = 2^-24 and u + 2 eta replaced by 1e-5, i.e. an error of
1e-5 relative to the sum of the magnitudes of the terms (the quantity the rounding error of any
summation is proportional to; a gradient element itself may cancel to nearly zero), and
E = 2^-24 sum_d |dout_d| |out_d| (the forward result and lse are fp32 numbers there).
"""
from __future__ import annotations

import numpy as np

from oracle import pskv_oracle as orc

F32_REL = 1e-5
BF16_ABS = 2e-2          # the stated bar
U_BF16 = 2.0 ** -8       # unit round-off of bf16
U_F32 = 2.0 ** -24
RMS_BAR = float(np.sqrt(2.0 / 3.0)) * U_BF16      # two independent roundings, mean square <= u^2/3 each
RMS_EXPECTED = 2.35e-3                            # the same with log-uniform mantissas (0.4247 u each)


def eta_fp32(nkeys: int) -> float:
    """Allowance for the fp32 arithmetic of the bf16 path, relative to the magnitude sums."""
    return nkeys * 2.0 ** -23 + 2.0 ** -16


def _abs_values(a: np.ndarray, dtype: str) -> np.ndarray:
    """|a| in the storage form of `dtype` (bf16: clear the sign bit)."""
    return (a & np.uint16(0x7FFF)) if dtype == "bf16" else np.abs(a)


class Ref(np.ndarray):
    """The oracle's result together with the magnitude sum A_d = sum_j w_j |V_jd| of every element
    (`mag`, same shape) and the largest number of keys a row sees (`nkeys`)."""

    def __new__(cls, out, mag, nkeys):
        obj = np.asarray(out).view(cls)
        obj.mag = mag
        obj.nkeys = nkeys
        return obj

    def __array_finalize__(self, obj):
        self.mag = getattr(obj, "mag", None)
        self.nkeys = getattr(obj, "nkeys", 0)


def oracle_out(inp: object, want_lse=False):
    """Oracle result (a Ref) of a single-prefix problem; with want_lse, (Ref, lse)."""
    dt = inp.w.dtype
    res = orc.attn(inp.q, inp.k_suf, inp.v_suf, inp.k_pre, inp.v_pre, inp.suf_len, inp.scale, dt, want_lse=want_lse)
    out, lse = res if want_lse else (res, None)
    mag = None
    if dt == "bf16":
        mag = orc.attn(inp.q, inp.k_suf, _abs_values(inp.v_suf, dt), inp.k_pre, _abs_values(inp.v_pre, dt), inp.suf_len,
                       inp.scale, dt)
    ref = Ref(out, mag, inp.w.P + inp.w.S)
    return (ref, lse) if want_lse else ref


def forward_bound(ref: Ref) -> np.ndarray:
    """F_d = (u + eta) A_d + u |out_d| for every element (bf16 path)."""
    return (U_BF16 + eta_fp32(ref.nkeys)) * ref.mag + U_BF16 * np.abs(np.asarray(ref))


def compare(got: np.ndarray, ref, suf_len: np.ndarray, dtype: str, what: str = ""):
    """got/ref: [B,S,Hq,D] float64 (ref a Ref for bf16). Returns a dict of error figures; asserts the bars."""
    B, S = ref.shape[:2]
    valid = np.arange(S)[None, :] < np.asarray(suf_len)[:, None]
    assert not np.isnan(got).any(), f"{what}: NaN in GPU output"
    assert np.all(got[~valid] == 0.0), f"{what}: padded rows must be exactly 0"
    r_all = np.asarray(ref)
    g, r = got[valid], r_all[valid]
    if g.size == 0:
        return {"n": 0}
    err = np.abs(g - r)
    res = {"n": int(g.size), "max_abs": float(err.max())}
    if dtype == "f32":
        rel = err / np.maximum(np.abs(r), 1e-300)
        res["max_rel"] = float(rel.max())
        assert res["max_rel"] <= F32_REL, f"{what}: max relative error {res['max_rel']:.3e} > {F32_REL}"
    else:
        assert isinstance(ref, Ref) and ref.mag is not None, "bf16 comparisons need the oracle's magnitude sums"
        sd = float(r.std())
        bound = forward_bound(ref)[valid]
        rms_ref = float(np.sqrt(np.mean(r * r)))
        res["std_ref"] = sd
        res["max_abs_over_std"] = float(err.max() / sd) if sd > 0 else 0.0      # printed, not a bar: see the header
        res["bound_ratio"] = float((err / np.maximum(bound, 1e-300)).max())
        res["rms_ratio"] = float(np.sqrt(np.mean(err * err)) / rms_ref) if rms_ref > 0 else 0.0
        assert res["max_abs"] <= BF16_ABS, f"{what}: max abs error {res['max_abs']:.3e} > {BF16_ABS}"
        assert res["bound_ratio"] <= 1.0, \
            f"{what}: |err| / ((u + eta) sum_j w_j|V_jd| + u|ref|) = {res['bound_ratio']:.3f} > 1"
        rms_bar = RMS_BAR + eta_fp32(ref.nkeys) * float(np.sqrt(np.mean(ref.mag[valid] ** 2))) / rms_ref
        assert res["rms_ratio"] <= rms_bar, f"{what}: rms error / rms(ref) = {res['rms_ratio']:.3e} > {rms_bar:.3e}"
    return res


def compare_lse(got: np.ndarray, ref: np.ndarray, suf_len: np.ndarray, dtype: str, what: str = "", nkeys: int = 0):
    """lse is an fp32 number on every path.  bf16 tensors (fp32 arithmetic): the row sum carries a
    relative error of at most eta, i.e. an absolute eta in its logarithm, plus the fp32 rounding
    of the scaled maximum and of the result (2^-22 |lse| together).  fp32 tensors (fp64 arithmetic): 1e-5."""
    B, Hq, S = ref.shape
    valid = np.broadcast_to((np.arange(S)[None, :] < np.asarray(suf_len)[:, None])[:, None, :], ref.shape)
    assert np.all(np.isneginf(got[~valid])), f"{what}: lse of padded rows must be -inf"
    if valid.any():
        err = np.abs(got[valid] - ref[valid])
        if dtype == "f32":
            tol = 1e-5 * np.maximum(1.0, np.abs(ref[valid]))
        else:
            tol = eta_fp32(nkeys if nkeys else 4096) + 2.0 ** -22 * np.abs(ref[valid])
        assert np.all(err <= tol), f"{what}: lse error {err.max():.3e}"


def oracle_out_multi(inp: object, want_lse=False):
    dt = inp.w.dtype
    res = orc.attn_multi(inp.q, inp.k_suf, inp.v_suf, inp.k_pre, inp.v_pre, inp.pre_len, inp.suf_len,
                         inp.scale, dt, want_lse=want_lse)
    out, lse = res if want_lse else (res, None)
    mag = None
    if dt == "bf16":
        mag = orc.attn_multi(inp.q, inp.k_suf, _abs_values(inp.v_suf, dt), inp.k_pre, _abs_values(inp.v_pre, dt),
                             inp.pre_len, inp.suf_len, inp.scale, dt)
    ref = Ref(out, mag, inp.w.P + inp.w.S)
    return (ref, lse) if want_lse else ref


LAMBDA = 9.0   # Hoeffding multiplier of the bound on |delta~ - delta|: fails with probability 2 exp(-LAMBDA^2/2) per row


class GradRef(np.ndarray):
    """An exact gradient (the oracle's) with its element-wise error bound (`bound`, the header's
    formula) and the bar on its rms error (`rms_bar`, absolute)."""

    def __new__(cls, val, bound, rms_bar):
        obj = np.asarray(val).view(cls)
        obj.bound = bound
        obj.rms_bar = rms_bar
        return obj

    def __array_finalize__(self, obj):
        self.bound = getattr(obj, "bound", None)
        self.rms_bar = getattr(obj, "rms_bar", None)


def _widen(a, dtype):
    """bf16 bit patterns (uint16) or fp32 values, widened exactly to float64."""
    if dtype == "bf16":
        return (np.ascontiguousarray(a, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return np.asarray(a, dtype=np.float64)


def grad_bounds(q, k_suf, v_suf, prefix_of, suf_len, dout64, scale, dtype):
    """The terms of the header's gradient bounds in float64 NumPy, for dq, dk_suf and dv_suf:
    returns three (rounding part, delta part, fp32 part) triples of arrays shaped like the gradients
    (padded rows 0), without the final u |gradient|.  prefix_of(b) -> (k_pre, v_pre) float64
    [P_b,Hkv,D]: candidate b's visible prefix rows."""
    q, k_suf, v_suf = (_widen(a, dtype) for a in (q, k_suf, v_suf))
    B, S, Hq, D = q.shape
    Hkv = k_suf.shape[2]
    G = Hq // Hkv
    parts = {n: [np.zeros(sh), np.zeros(sh), np.zeros(sh)] for n, sh in (("q", q.shape), ("k", k_suf.shape), ("v", v_suf.shape))}
    bf16 = dtype == "bf16"
    for b in range(B):
        n = int(suf_len[b])
        if n == 0:
            continue
        kp, vp = prefix_of(b)
        P = kp.shape[0]
        u = U_BF16 if bf16 else U_F32
        eta = eta_fp32(P + n) if bf16 else 0.5 * (F32_REL - U_F32)
        K = np.concatenate([kp, k_suf[b, :n]], axis=0).transpose(1, 0, 2)           # [Hkv,P+n,D]
        V = np.concatenate([vp, v_suf[b, :n]], axis=0).transpose(1, 0, 2)
        Q = q[b, :n].transpose(1, 0, 2).reshape(Hkv, G, n, D)                       # [Hkv,G,n,D]
        dO = np.nan_to_num(dout64[b, :n]).transpose(1, 0, 2).reshape(Hkv, G, n, D)
        s = np.einsum("kgid,kjd->kgij", Q, K) * scale
        vis = np.arange(P + n)[None, :] <= P + np.arange(n)[:, None]                # prefix + causal
        s = np.where(vis, s, -np.inf)
        p = np.exp(s - s.max(axis=-1, keepdims=True))
        p /= p.sum(axis=-1, keepdims=True)
        out = np.einsum("kgij,kjd->kgid", p, V)
        dp = np.einsum("kgid,kjd->kgij", dO, V)
        delta = (p * dp).sum(axis=-1, keepdims=True)
        ads = p * np.abs(dp - delta)                                                # |ds_j|
        aK, aQ, adO, aV = np.abs(K), np.abs(Q), np.abs(dO), np.abs(V)
        if bf16:
            E = LAMBDA * u * np.sqrt((p * p * dp * dp).sum(axis=-1) + (dO * dO * out * out).sum(axis=-1))    # [Hkv,G,n]
        else:
            E = U_F32 * (adO * np.abs(out)).sum(axis=-1)
        # fp32 noise of <dout,V_j> and of <dout,out>, which cancel in dp_j - delta
        Cj = eta * (np.einsum("kgid,kjd->kgij", adO, aV) + (adO * np.abs(out)).sum(axis=-1)[..., None])
        w_round = u * ads                                                           # the rounding of ds to bf16
        w_delta = (1 + u) * p * E[..., None]
        w_fp32 = 2 * eta * ads + (1 + u) * p * Cj
        for part, wq in enumerate((w_round, w_delta, w_fp32)):
            parts["q"][part][b, :n] = (scale * np.einsum("kgij,kjd->kgid", wq, aK)).reshape(Hq, n, D).transpose(1, 0, 2)
            parts["k"][part][b, :n] = (scale * np.einsum("kgij,kgid->kjd", wq[..., P:], aQ)).transpose(1, 0, 2)
        parts["v"][0][b, :n] = (u * np.einsum("kgij,kgid->kjd", p[..., P:], adO)).transpose(1, 0, 2)
        parts["v"][2][b, :n] = (2 * eta * np.einsum("kgij,kgid->kjd", p[..., P:], adO)).transpose(1, 0, 2)
    return parts["q"], parts["k"], parts["v"]


def _finish_grad(val, parts, valid_rows, dtype):
    """Element-wise bound = rounding + delta + fp32 parts + u |value|; rms bar as in the header."""
    rnd, dlt, f32p = parts
    u = U_BF16 if dtype == "bf16" else U_F32
    bound = rnd + dlt + f32p + u * np.abs(val)

    def rms(a):
        a = a[valid_rows]
        return float(np.sqrt(np.mean(a * a))) if a.size else 0.0

    rms_bar = float(np.sqrt(2.0 / 3.0)) * u * rms(val) + rms(dlt) / (np.sqrt(3.0) * LAMBDA) + rms(f32p)
    return GradRef(val, bound, rms_bar)


def oracle_bwd(inp, dout64):
    """The oracle's gradients (dq, dk_suf, dv_suf) of a single-prefix problem as GradRefs."""
    w = inp.w
    dt = w.dtype
    kp = inp.k_pre if w.P > 0 else np.zeros((0, w.Hkv, w.D), dtype=inp.q.dtype)
    vp = inp.v_pre if w.P > 0 else np.zeros((0, w.Hkv, w.D), dtype=inp.q.dtype)
    d0 = np.nan_to_num(dout64, nan=0.0)
    grads = orc.attn_bwd(inp.q, inp.k_suf, inp.v_suf, kp, vp, inp.suf_len, d0, inp.scale, dt)
    kp64, vp64 = _widen(kp, dt), _widen(vp, dt)
    parts = grad_bounds(inp.q, inp.k_suf, inp.v_suf, lambda b: (kp64, vp64), inp.suf_len, d0, inp.scale, dt)
    valid = np.arange(w.S)[None, :] < np.asarray(inp.suf_len)[:, None]
    return tuple(_finish_grad(g, pt, valid, dt) for g, pt in zip(grads, parts))


def oracle_bwd_multi(inp, dout64):
    """The same for the multi-instruction form: candidate b sees the real rows of its instruction's prefix."""
    w = inp.w
    dt = w.dtype
    d0 = np.nan_to_num(dout64, nan=0.0)
    grads = orc.attn_bwd_multi(inp.q, inp.k_suf, inp.v_suf, inp.k_pre, inp.v_pre, inp.pre_len, inp.suf_len, d0,
                               inp.scale, dt)
    kp64, vp64 = _widen(inp.k_pre, dt), _widen(inp.v_pre, dt)

    def prefix_of(b):
        n = b // w.C
        pl = min(max(int(inp.pre_len[n]), 0), w.P)
        return kp64[n, w.P - pl:], vp64[n, w.P - pl:]

    parts = grad_bounds(inp.q, inp.k_suf, inp.v_suf, prefix_of, inp.suf_len, d0, inp.scale, dt)
    valid = np.arange(w.S)[None, :] < np.asarray(inp.suf_len)[:, None]
    return tuple(_finish_grad(g, pt, valid, dt) for g, pt in zip(grads, parts))


def compare_grad(got, ref, valid_rows, dtype, what):
    """One gradient tensor [B,S,H,D] against the oracle's (a GradRef): padded rows exactly zero, every
    valid element inside its bound, the rms error inside its bar."""
    assert isinstance(ref, GradRef) and ref.bound is not None, "gradient comparisons need the element-wise bounds"
    assert not np.isnan(got).any(), f"{what}: NaN"
    assert np.all(got[~valid_rows] == 0.0), f"{what}: padded rows must be exactly 0"
    g, r, bound = got[valid_rows], np.asarray(ref)[valid_rows], ref.bound[valid_rows]
    if g.size == 0:
        return {"n": 0}
    err = np.abs(g - r)
    res = {"n": int(g.size), "max_abs": float(err.max())}
    res["bound_ratio"] = float((err / np.maximum(bound, 1e-300)).max())
    rms_ref = float(np.sqrt(np.mean(r * r)))
    rms_err = float(np.sqrt(np.mean(err * err)))
    res["rms_ratio"] = rms_err / rms_ref if rms_ref > 0 else 0.0
    res["rms_over_bar"] = rms_err / ref.rms_bar if ref.rms_bar > 0 else 0.0
    assert res["bound_ratio"] <= 1.0, f"{what}: |err| / bound = {res['bound_ratio']:.3f} > 1"
    assert rms_err <= ref.rms_bar, f"{what}: rms error {rms_err:.3e} > {ref.rms_bar:.3e}"
    return res
