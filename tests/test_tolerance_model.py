"""CPU checks of the error bounds the GPU parity tests assert (tests/parity_util.py): the kernels'
rounding points are emulated in NumPy on the oracle's exact softmax weights - weights to bf16 before
the value product, denominator from the unrounded weights, one bf16 store; in the backward pass
delta from the stored bf16 result, ds and p to bf16 before the second products - and the emulated
results must (a) sit inside the element-wise bounds, (b) show the rms error the model predicts, while
(c) results with a planted mistake of the size the bounds are meant to catch must fail.  No GPU and
no value from the HIP path is involved."""
import numpy as np
import pytest

from oracle import pskv_oracle as orc
from paper_2603_13420_amd import inputs as gen
import parity_util as pu


def rne_bf16(x):
    return gen.bf16_bits_to_f32(gen.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))).astype(np.float64)


def emulate_forward(inp):
    """Eq. 2 with the matrix-core kernels' rounding points, from the oracle's exact weights."""
    w = inp.w
    out, lse, probs = orc.attn(inp.q, inp.k_suf, inp.v_suf, inp.k_pre, inp.v_pre, inp.suf_len, inp.scale, w.dtype,
                               want_lse=True, want_probs=True)
    G = w.Hq // w.Hkv
    vp, vs = inp.as_f32("v_pre").astype(np.float64), inp.as_f32("v_suf").astype(np.float64)
    emu = np.zeros_like(out)
    for b in range(w.B):
        n = int(inp.suf_len[b])
        for h in range(w.Hq):
            V = np.concatenate([vp[:, h // G], vs[b, :n, h // G]], axis=0)
            for i in range(n):
                pr = probs[b, h, i, :w.P + i + 1].copy()
                pr[w.P:] = probs[b, h, i, w.P:w.P + i + 1]
                # unnormalised weights relative to the first tile's maximum (any reference gives the same statistics)
                e = pr / pr[:min(32, len(pr))].max()
                emu[b, i, h] = rne_bf16((rne_bf16(e) @ V[:len(e)]) / e.sum())
    return out, lse, probs, emu


CASES = [(4, 256, 24, 16, 24, 8, 2), (3, 0, 24, 1, 24, 4, 1), (2, 130, 40, 30, 40, 4, 4)]


@pytest.mark.parametrize("B,P,S,lo,hi,Hq,Hkv", CASES)
def test_forward_bound_holds_for_the_emulated_roundings(B, P, S, lo, hi, Hq, Hkv):
    wl = gen.custom_workload("tolfwd", B, P, S, lo, hi, Hq, Hkv, 128, "bf16", index=3000 + P)
    inp = gen.make_inputs(wl, pad="nan")
    if P == 0:
        inp = gen.Inputs(wl, inp.q, inp.k_suf, inp.v_suf, np.zeros((0, Hkv, 128), np.uint16), np.zeros((0, Hkv, 128), np.uint16),
                         inp.suf_len, inp.scale)
    out, _, _, emu = emulate_forward(inp)
    ref = pu.oracle_out(inp)
    assert np.array_equal(np.asarray(ref), out)
    res = pu.compare(emu, ref, inp.suf_len, "bf16", "emulated forward")
    assert res["bound_ratio"] <= 1.0
    # the prediction for independent roundings with log-uniform mantissas: 2.35e-3 rms(ref) (rows that see
    # a handful of keys fall below it: their largest weight is exactly one and is not rounded at all)
    assert res["rms_ratio"] <= 1.25 * pu.RMS_EXPECTED, res
    if P >= 100:
        assert 0.75 * pu.RMS_EXPECTED <= res["rms_ratio"], res
    valid = np.arange(S)[None, :] < inp.suf_len[:, None]
    # planted mistakes: a relative error of 2 u everywhere; one weight-rounding too many (weights rounded
    # twice over: the sum taken from the rounded weights as well, all of them rounded down)
    with pytest.raises(AssertionError):
        pu.compare(np.where(valid[..., None, None], np.asarray(ref) * (1 + 2 * pu.U_BF16), 0.0), ref, inp.suf_len, "bf16", "planted")
    with pytest.raises(AssertionError):
        pu.compare(np.where(valid[..., None, None], np.asarray(ref) + 1.5 * pu.forward_bound(ref), 0.0), ref, inp.suf_len,
                   "bf16", "planted")
    # an error pattern that stays inside the element-wise bound but is systematic (every element off by 60 %
    # of its bound) is caught by the rms bar
    with pytest.raises(AssertionError):
        pu.compare(np.where(valid[..., None, None], np.asarray(ref) + 0.6 * pu.forward_bound(ref), 0.0), ref, inp.suf_len,
                   "bf16", "planted")


def emulate_backward(inp, dout64, out_stored, lse):
    """The gradients with the kernels' rounding points: delta from the stored (bf16) forward result,
    ds and p rounded to bf16 before the second products, one bf16 store per gradient."""
    w = inp.w
    q, ks, vs = (inp.as_f32(n).astype(np.float64) for n in ("q", "k_suf", "v_suf"))
    kp, vp = (inp.as_f32(n).astype(np.float64) for n in ("k_pre", "v_pre"))
    G = w.Hq // w.Hkv
    dq, dk, dv = np.zeros(q.shape), np.zeros(ks.shape), np.zeros(vs.shape)
    for b in range(w.B):
        n = int(inp.suf_len[b])
        for h in range(w.Hq):
            k = h // G
            K = np.concatenate([kp[:, k], ks[b, :n, k]], axis=0)
            V = np.concatenate([vp[:, k], vs[b, :n, k]], axis=0)
            for i in range(n):
                nv = w.P + i + 1
                s = (K[:nv] @ q[b, i, h]) * inp.scale
                p = np.exp(s - lse[b, h, i])
                dp = V[:nv] @ dout64[b, i, h]
                delta = float(dout64[b, i, h] @ out_stored[b, i, h])
                ds = rne_bf16(p * (dp - delta))
                dq[b, i, h] = inp.scale * (ds @ K[:nv])
                dk[b, :i + 1, k] += inp.scale * ds[w.P:, None] * q[b, i, h][None, :]
                dv[b, :i + 1, k] += rne_bf16(p[w.P:])[:, None] * dout64[b, i, h][None, :]
    return rne_bf16(dq), rne_bf16(dk), rne_bf16(dv)


@pytest.mark.parametrize("B,P,S,lo,hi,Hq,Hkv", CASES)
def test_gradient_bounds_hold_for_the_emulated_roundings(B, P, S, lo, hi, Hq, Hkv):
    wl = gen.custom_workload("tolbwd", B, P, S, lo, hi, Hq, Hkv, 128, "bf16", index=3100 + P)
    inp = gen.make_inputs(wl, pad="nan")
    if P == 0:
        inp = gen.Inputs(wl, inp.q, inp.k_suf, inp.v_suf, np.zeros((0, Hkv, 128), np.uint16), np.zeros((0, Hkv, 128), np.uint16),
                         inp.suf_len, inp.scale)
    _, lse, _, emu_out = emulate_forward(inp)
    _, dout64 = pu.make_dout(inp, 77)
    d0 = np.nan_to_num(dout64, nan=0.0)
    got = emulate_backward(inp, d0, emu_out, lse)
    refs = pu.oracle_bwd(inp, dout64)
    valid = np.arange(S)[None, :] < inp.suf_len[:, None]
    for name, g, r in zip(("dq", "dk_suf", "dv_suf"), got, refs):
        g = np.where(valid[..., None, None], g, 0.0)
        res = pu.compare_grad(g, r, valid, "bf16", f"emulated {name}")
        print(name, res)
        assert res["bound_ratio"] <= 1.0 and res["rms_over_bar"] <= 1.0
        # planted mistakes: one more bf16 rounding error everywhere; delta left out of ds (dq, dk)
        with pytest.raises(AssertionError):
            pu.compare_grad(np.where(valid[..., None, None], np.asarray(r) + 1.5 * r.bound, 0.0), r, valid, "bf16", "planted")
        with pytest.raises(AssertionError):
            pu.compare_grad(np.where(valid[..., None, None], np.asarray(r) + 0.6 * r.bound, 0.0), r, valid, "bf16", "planted")
    # delta taken from a forward result whose every element is off by 2^-5 of itself, the errors lined up with
    # the signs of dout (what a forward pass that loses two more bits would hand over): dq must fail
    bad = emulate_backward(inp, d0, emu_out + 2.0 ** -5 * np.abs(emu_out) * np.sign(d0), lse)
    with pytest.raises(AssertionError):
        pu.compare_grad(np.where(valid[..., None, None], bad[0], 0.0), refs[0], valid, "bf16", "planted delta")


def test_fp32_gradient_bound_is_relative_to_the_magnitude_of_the_terms():
    wl = gen.custom_workload("tolf32", 3, 20, 9, 1, 9, 4, 2, 64, "f32", index=3200)
    inp = gen.make_inputs(wl, pad="nan")
    _, dout64 = pu.make_dout(inp, 78)
    refs = pu.oracle_bwd(inp, dout64)
    valid = np.arange(wl.S)[None, :] < inp.suf_len[:, None]
    for r in refs:
        v = np.asarray(r)[valid]
        bd = r.bound[valid]
        assert np.all(bd >= pu.U_F32 * np.abs(v))
        # the oracle's own result rounded to fp32 passes; an error of 1e-4 of the element's magnitude sum does not
        g32 = np.where(valid[..., None, None], np.asarray(r).astype(np.float32).astype(np.float64), 0.0)
        pu.compare_grad(g32, r, valid, "f32", "fp32 rounding")
        with pytest.raises(AssertionError):
            pu.compare_grad(np.where(valid[..., None, None], np.asarray(r) + 12 * r.bound, 0.0), r, valid, "f32", "planted")
