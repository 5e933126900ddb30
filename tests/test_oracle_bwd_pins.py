"""Pins for the backward oracle (gradient with respect to the suffix side; the prefix K/V is a
constant): finite differences of the already pinned forward oracle, a library's automatic
differentiation of a plain forward, and structural facts of the softmax gradient."""
import math

import numpy as np
import pytest
import torch

from oracle import pskv_oracle as orc


def problem(rng, B, P, S, Hq, Hkv, D):
    q = rng.standard_normal((B, S, Hq, D))
    ks = rng.standard_normal((B, S, Hkv, D))
    vs = rng.standard_normal((B, S, Hkv, D))
    kp = rng.standard_normal((P, Hkv, D))
    vp = rng.standard_normal((P, Hkv, D))
    sl = rng.integers(0, S + 1, size=B).astype(np.int32)
    sl[0] = S
    do = rng.standard_normal((B, S, Hq, D))
    return q, ks, vs, kp, vp, sl, do


@pytest.mark.parametrize("B,P,S,Hq,Hkv,D", [(2, 3, 3, 2, 1, 3), (2, 0, 3, 2, 2, 2), (1, 4, 2, 4, 2, 3)])
def test_central_differences_of_the_forward_oracle(B, P, S, Hq, Hkv, D):
    rng = np.random.default_rng(20 + B + P)
    q, ks, vs, kp, vp, sl, do = problem(rng, B, P, S, Hq, Hkv, D)
    scale = 1.0 / math.sqrt(D)
    dq, dk, dv = orc.attn_bwd(q, ks, vs, kp, vp, sl, do, scale, "f64")

    def loss(q_, ks_, vs_):
        return float((do * orc.attn(q_, ks_, vs_, kp, vp, sl, scale, "f64")).sum())

    eps = 1e-6
    for name, grad, idx in (("q", dq, 0), ("k", dk, 1), ("v", dv, 2)):
        args = [q, ks, vs]
        base = args[idx]
        num = np.zeros_like(base)
        it = np.nditer(base, flags=["multi_index"])
        for _ in it:
            mi = it.multi_index
            hi, lo = base.copy(), base.copy()
            hi[mi] += eps
            lo[mi] -= eps
            a_hi, a_lo = list(args), list(args)
            a_hi[idx], a_lo[idx] = hi, lo
            num[mi] = (loss(*a_hi) - loss(*a_lo)) / (2 * eps)
        np.testing.assert_allclose(grad, num, rtol=0, atol=2e-8, err_msg=name)


def test_library_autodiff_of_a_plain_forward():
    """torch autograd through an ordinary masked softmax attention written with library ops."""
    rng = np.random.default_rng(31)
    B, P, S, Hq, Hkv, D = 3, 6, 5, 4, 2, 8
    q, ks, vs, kp, vp, sl, do = problem(rng, B, P, S, Hq, Hkv, D)
    scale = 0.3
    dq, dk, dv = orc.attn_bwd(q, ks, vs, kp, vp, sl, do, scale, "f64")
    G = Hq // Hkv
    tq, tks, tvs = (torch.tensor(x, requires_grad=True) for x in (q, ks, vs))
    tkp, tvp, tdo = torch.tensor(kp), torch.tensor(vp), torch.tensor(do)
    total = torch.zeros((), dtype=torch.float64)
    for b in range(B):
        L = int(sl[b])
        if L == 0:
            continue
        K = torch.cat([tkp, tks[b, :L]], dim=0).permute(1, 0, 2).repeat_interleave(G, dim=0)   # [Hq, P+L, D]
        V = torch.cat([tvp, tvs[b, :L]], dim=0).permute(1, 0, 2).repeat_interleave(G, dim=0)
        Q = tq[b, :L].permute(1, 0, 2)
        s = (Q @ K.transpose(1, 2)) * scale
        col, row = torch.arange(P + L)[None, :], torch.arange(L)[:, None]
        s = s.masked_fill(~(col <= P + row)[None], float("-inf"))
        o = torch.softmax(s, dim=-1) @ V                                                        # [Hq, L, D]
        total = total + (o.permute(1, 0, 2) * tdo[b, :L]).sum()
    total.backward()
    np.testing.assert_allclose(dq, tq.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dk, tks.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dv, tvs.grad.numpy(), rtol=0, atol=1e-12)


def test_structure_of_the_gradient():
    rng = np.random.default_rng(32)
    B, P, S, Hq, Hkv, D = 3, 5, 4, 4, 2, 6
    q, ks, vs, kp, vp, sl, do = problem(rng, B, P, S, Hq, Hkv, D)
    sl[:] = [4, 2, 0]
    dq, dk, dv = orc.attn_bwd(q, ks, vs, kp, vp, sl, do, 0.4, "f64")
    # padded rows receive exactly nothing; a candidate without suffix has no gradient at all
    assert (dq[1, 2:] == 0).all() and (dk[1, 2:] == 0).all() and (dv[1, 2:] == 0).all()
    assert (dq[2] == 0).all() and (dk[2] == 0).all() and (dv[2] == 0).all()
    # dout on padded rows does not matter, and candidates do not influence one another
    do2 = do.copy()
    do2[1, 2:] = 1e6
    do2[2] = -1e6
    again = orc.attn_bwd(q, ks, vs, kp, vp, sl, do2, 0.4, "f64")
    assert all(np.array_equal(a, b) for a, b in zip((dq, dk, dv), again))
    q3 = q.copy()
    q3[0] += 1.0
    other = orc.attn_bwd(q3, ks, vs, kp, vp, sl, do, 0.4, "f64")
    assert np.array_equal(other[0][1:], dq[1:]) and np.array_equal(other[1][1:], dk[1:])
    # dV of the last suffix row only sees the last query row of each head: p_last * dout_last
    out, probs = orc.attn(q, ks, vs, kp, vp, sl, 0.4, "f64", want_probs=True)
    G = Hq // Hkv
    for k in range(Hkv):
        want = sum(probs[0, k * G + g, 3, P + 3] * do[0, 3, k * G + g] for g in range(G))
        np.testing.assert_allclose(dv[0, 3, k], want, rtol=0, atol=1e-13)
    # the loss is linear in dout and the forward output is linear in v: sum(dv * v_suf) plus the
    # prefix share equals the loss, so with an empty prefix  sum(dv * v_suf) == sum(dout * out)
    nop = np.zeros((0, Hkv, D))
    out0 = orc.attn(q, ks, vs, nop, nop, sl, 0.4, "f64")
    _, _, dv0 = orc.attn_bwd(q, ks, vs, nop, nop, sl, do, 0.4, "f64")
    np.testing.assert_allclose((dv0 * vs).sum(), (do * out0).sum(), rtol=1e-12)
    # with an empty prefix the scores depend on q and k_suf only through products q.k, so the loss
    # is unchanged under (q -> t q, k_suf -> k_suf / t); differentiating at t = 1 (Euler's relation)
    # gives  sum(dq * q) == sum(dk * k_suf)
    dq0, dk0, _ = orc.attn_bwd(q, ks, vs, nop, nop, sl, do, 0.4, "f64")
    np.testing.assert_allclose((dq0 * q).sum(), (dk0 * ks).sum(), rtol=1e-10, atol=1e-12)


def test_bf16_inputs_are_widened_exactly():
    from paper_2603_13420_amd import inputs as gen
    rng = np.random.default_rng(33)
    q, ks, vs, kp, vp, sl, do = problem(rng, 2, 4, 3, 2, 1, 8)
    bits = [gen.f32_to_bf16_bits(x.astype(np.float32)) for x in (q, ks, vs, kp, vp)]
    wide = [gen.bf16_bits_to_f32(b).astype(np.float64) for b in bits]
    a = orc.attn_bwd(*bits, sl, do, 0.35, "bf16")
    b = orc.attn_bwd(*wide, sl, do, 0.35, "f64")
    assert all(np.array_equal(x, y) for x, y in zip(a, b))


def multi_problem(rng, Np, C, Pp, S, Hq, Hkv, D):
    B = Np * C
    q = rng.standard_normal((B, S, Hq, D))
    ks = rng.standard_normal((B, S, Hkv, D))
    vs = rng.standard_normal((B, S, Hkv, D))
    kp = rng.standard_normal((Np, Pp, Hkv, D))
    vp = rng.standard_normal((Np, Pp, Hkv, D))
    pl = rng.integers(0, Pp + 1, size=Np).astype(np.int32)
    pl[0] = Pp
    sl = rng.integers(0, S + 1, size=B).astype(np.int32)
    sl[0] = S
    do = rng.standard_normal((B, S, Hq, D))
    return q, ks, vs, kp, vp, pl, sl, do


def test_multi_instruction_backward_is_the_derivative_of_the_multi_instruction_forward():
    """Central differences of the (separately pinned) multi-instruction forward oracle, including
    with respect to prefix padding rows, which must not matter."""
    rng = np.random.default_rng(77)
    Np, C, Pp, S, Hq, Hkv, D = 3, 2, 4, 3, 2, 1, 3
    q, ks, vs, kp, vp, pl, sl, do = multi_problem(rng, Np, C, Pp, S, Hq, Hkv, D)
    pl[1] = 0
    scale = 0.7
    dq, dk, dv = orc.attn_bwd_multi(q, ks, vs, kp, vp, pl, sl, do, scale, "f64")

    def loss(q_, ks_, vs_):
        return float((do * orc.attn_multi(q_, ks_, vs_, kp, vp, pl, sl, scale, "f64")).sum())

    eps = 1e-6
    for name, grad, idx in (("q", dq, 0), ("k", dk, 1), ("v", dv, 2)):
        args = [q, ks, vs]
        base = args[idx]
        num = np.zeros_like(base)
        it = np.nditer(base, flags=["multi_index"])
        for _ in it:
            mi = it.multi_index
            hi, lo = base.copy(), base.copy()
            hi[mi] += eps
            lo[mi] -= eps
            a_hi, a_lo = list(args), list(args)
            a_hi[idx], a_lo[idx] = hi, lo
            num[mi] = (loss(*a_hi) - loss(*a_lo)) / (2 * eps)
        np.testing.assert_allclose(grad, num, rtol=0, atol=2e-8, err_msg=name)
    # what lies in the left padding of a prefix reaches no gradient
    kp2, vp2 = kp.copy(), vp.copy()
    for n in range(Np):
        kp2[n, :Pp - pl[n]] = np.nan
        vp2[n, :Pp - pl[n]] = np.nan
    for a_, b_ in zip((dq, dk, dv), orc.attn_bwd_multi(q, ks, vs, kp2, vp2, pl, sl, do, scale, "f64")):
        assert np.array_equal(a_, b_)


def test_multi_instruction_backward_with_one_instruction_is_the_single_prefix_backward():
    rng = np.random.default_rng(78)
    q, ks, vs, kp, vp, sl, do = problem(rng, 3, 5, 4, 4, 2, 4)
    one = orc.attn_bwd(q, ks, vs, kp, vp, sl, do, 0.5, "f64")
    multi = orc.attn_bwd_multi(q, ks, vs, kp[None], vp[None], None, sl, do, 0.5, "f64")
    for a_, b_ in zip(one, multi):
        assert np.array_equal(a_, b_)
