"""Pins for the CPU oracle: what the paper's definitions and the mathematics fix.

Each test is chosen so that a plausible slip in the oracle (dropped term, wrong mask index,
K/V swapped, wrong GQA map, missing scale) fails at least one of them.  None of them calls
the HIP path.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import pskv_oracle as orc
from paper_2603_13420_amd import inputs as gen

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rand_problem(rng, B, P, S, Hq, Hkv, D, ragged=True):
    q = rng.standard_normal((B, S, Hq, D))
    ks = rng.standard_normal((B, S, Hkv, D))
    vs = rng.standard_normal((B, S, Hkv, D))
    kp = rng.standard_normal((P, Hkv, D))
    vp = rng.standard_normal((P, Hkv, D))
    sl = rng.integers(0 if ragged else S, S + 1, size=B).astype(np.int32)
    return q, ks, vs, kp, vp, sl


def brute_force(q, ks, vs, kp, vp, sl, scale):
    """Independent scalar implementation: no duplication, no concatenation, different loop
    order (d outermost for the output), exact summation with math.fsum."""
    B, S, Hq, D = q.shape
    Hkv = ks.shape[2]
    P = kp.shape[0]
    G = Hq // Hkv
    out = np.zeros((B, S, Hq, D))
    lse = np.full((B, Hq, S), -np.inf)
    for h in range(Hq):
        kv = h // G
        for b in range(B):
            for i in range(int(sl[b])):
                sc_pre = [scale * math.fsum(q[b, i, h, d] * kp[j, kv, d] for d in range(D))
                          for j in range(P)]
                sc_suf = [scale * math.fsum(q[b, i, h, d] * ks[b, t, kv, d] for d in range(D))
                          for t in range(i + 1)]
                mx = max(sc_pre + sc_suf)
                w_pre = [math.exp(s - mx) for s in sc_pre]
                w_suf = [math.exp(s - mx) for s in sc_suf]
                z = math.fsum(w_pre + w_suf)
                for d in range(D):
                    out[b, i, h, d] = (math.fsum(w * vp[j, kv, d] for j, w in enumerate(w_pre)) +
                                       math.fsum(w * vs[b, t, kv, d] for t, w in enumerate(w_suf))) / z
                lse[b, h, i] = mx + math.log(z)
    return out, lse


@pytest.mark.parametrize("B,P,S,Hq,Hkv,D", [(3, 5, 4, 2, 1, 4), (2, 0, 3, 2, 2, 3), (1, 7, 1, 3, 1, 2),
                                            (2, 3, 4, 6, 2, 5)])
def test_brute_force_tiny(B, P, S, Hq, Hkv, D):
    rng = np.random.default_rng(100 + B + P)
    q, ks, vs, kp, vp, sl = rand_problem(rng, B, P, S, Hq, Hkv, D)
    scale = 0.37
    out, lse = orc.attn(q, ks, vs, kp, vp, sl, scale, "f64", want_lse=True)
    ref, ref_lse = brute_force(q, ks, vs, kp, vp, sl, scale)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)
    valid = np.arange(S)[None, None, :] < sl[:, None, None]
    valid = np.broadcast_to(valid, lse.shape)
    np.testing.assert_allclose(lse[valid], ref_lse[valid], rtol=0, atol=1e-12)
    assert np.all(np.isneginf(lse[~valid]))
    out_np, lse_np = orc.attn_numpy(q, ks, vs, kp, vp, sl, scale, "f64")
    np.testing.assert_allclose(out_np, ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse_np[valid], ref_lse[valid], rtol=0, atol=1e-12)


def test_handworked_golden():
    """tests/golden/handworked_ln2.txt: every weight is a power of two, results are rationals."""
    L = math.log(2.0)
    nan = float("nan")
    q = np.array([[[L, 0.0], [0.0, 2 * L]], [[-L, L], [nan, nan]]]).reshape(2, 2, 1, 2)
    ks = np.array([[[1.0, 1.0], [3.0, -1.0]], [[0.0, -1.0], [nan, nan]]]).reshape(2, 2, 1, 2)
    vs = np.array([[[4.0, -2.0], [8.0, 8.0]], [[6.0, 3.0], [nan, nan]]]).reshape(2, 2, 1, 2)
    kp = np.array([[1.0, 0.0], [0.0, 1.0]]).reshape(2, 1, 2)
    vp = np.array([[1.0, 0.0], [0.0, 1.0]]).reshape(2, 1, 2)
    sl = np.array([2, 1], dtype=np.int32)
    out, lse = orc.attn(q, ks, vs, kp, vp, sl, 1.0, "f64", want_lse=True)
    rows = [l.split() for l in open(os.path.join(GOLD, "handworked_ln2.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 4
    for r in rows:
        b, i = int(r[0]), int(r[1])
        o0, o1, z = (Fraction(int(r[2]), int(r[3])), Fraction(int(r[4]), int(r[5])),
                     Fraction(int(r[6]), int(r[7])))
        assert abs(out[b, i, 0, 0] - float(o0)) < 1e-14
        assert abs(out[b, i, 0, 1] - float(o1)) < 1e-14
        if z == 0:
            assert np.isneginf(lse[b, 0, i])
        else:
            assert abs(math.exp(lse[b, 0, i]) - float(z)) < 1e-13


@pytest.mark.parametrize("P,n,D", [(9, 6, 8), (0, 5, 4), (17, 1, 16)])
def test_single_candidate_is_plain_causal_attention(P, n, D):
    """B = 1: the candidate's rows are the last n rows of ordinary causal attention over the
    concatenation prefix + suffix (the paper's No-Cache / Standard-KV / PSKV equivalence,
    App. D), computed here by the library routine on CPU in float64."""
    rng = np.random.default_rng(7 + P)
    H = 3
    x_q = rng.standard_normal((P + n, H, D))      # queries for all positions (prefix ones unused)
    x_k = rng.standard_normal((P + n, H, D))
    x_v = rng.standard_normal((P + n, H, D))
    tq = torch.from_numpy(x_q).permute(1, 0, 2)[None]   # [1,H,T,D]
    tk = torch.from_numpy(x_k).permute(1, 0, 2)[None]
    tv = torch.from_numpy(x_v).permute(1, 0, 2)[None]
    full = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
    ref = full[0].permute(1, 0, 2).numpy()[P:]          # [n,H,D]
    out = orc.attn(x_q[None, P:], x_k[None, P:], x_v[None, P:], x_k[:P], x_v[:P],
                   np.array([n], dtype=np.int32), 1.0 / math.sqrt(D), "f64")
    np.testing.assert_allclose(out[0], ref, rtol=0, atol=1e-12)


def test_softmax_rows_sum_to_one_and_mask_is_exact():
    rng = np.random.default_rng(3)
    B, P, S, Hq, Hkv, D = 4, 6, 5, 4, 2, 8
    q, ks, vs, kp, vp, sl = rand_problem(rng, B, P, S, Hq, Hkv, D)
    sl[0] = S
    sl[1] = 0
    out, probs = orc.attn(q, ks, vs, kp, vp, sl, 0.5, "f64", want_probs=True)
    assert probs.shape == (B, Hq, S, P + S)
    assert np.all(probs >= 0)
    for b in range(B):
        for i in range(S):
            row = probs[b, :, i, :]
            if i < sl[b]:
                np.testing.assert_allclose(row.sum(axis=-1), 1.0, rtol=0, atol=1e-12)
                assert np.all(row[:, :P + i + 1] > 0)
                assert np.all(row[:, P + i + 1:] == 0.0)      # future and padded keys: exactly 0
            else:
                assert np.all(row == 0.0)
                assert np.all(out[b, i] == 0.0)


def test_batch_composition_invariance_bitwise():
    """A candidate's output does not depend on which other candidates share its batch
    (each one only ever sees the prefix and itself): permute, drop, and change the others."""
    rng = np.random.default_rng(11)
    B, P, S, Hq, Hkv, D = 6, 10, 7, 4, 2, 8
    q, ks, vs, kp, vp, sl = rand_problem(rng, B, P, S, Hq, Hkv, D)
    sl[2] = S
    base = orc.attn(q, ks, vs, kp, vp, sl, 0.3, "f64")
    perm = rng.permutation(B)
    out_p = orc.attn(q[perm], ks[perm], vs[perm], kp, vp, sl[perm], 0.3, "f64")
    assert np.array_equal(out_p, base[perm])
    keep = np.array([4, 2])
    out_k = orc.attn(q[keep], ks[keep], vs[keep], kp, vp, sl[keep], 0.3, "f64")
    assert np.array_equal(out_k, base[keep])
    q2, ks2, vs2, sl2 = q.copy(), ks.copy(), vs.copy(), sl.copy()
    others = [b for b in range(B) if b != 2]
    q2[others] += 1.0
    ks2[others] *= -2.0
    vs2[others] = 5.0
    sl2[others] = rng.integers(0, S + 1, size=len(others))
    out_c = orc.attn(q2, ks2, vs2, kp, vp, sl2, 0.3, "f64")
    assert np.array_equal(out_c[2], base[2])


def test_closed_forms():
    rng = np.random.default_rng(5)
    B, P, S, Hq, Hkv, D = 3, 7, 4, 2, 2, 6
    q, ks, vs, kp, vp, sl = rand_problem(rng, B, P, S, Hq, Hkv, D, ragged=False)
    # (a) all keys equal -> uniform weights -> running mean of the visible V rows
    kvec = rng.standard_normal((Hkv, D))
    ks_e = np.broadcast_to(kvec, ks.shape).copy()
    kp_e = np.broadcast_to(kvec, kp.shape).copy()
    out = orc.attn(q, ks_e, vs, kp_e, vp, sl, 0.4, "f64")
    for b in range(B):
        for i in range(S):
            for h in range(Hq):
                want = (vp[:, h].sum(0) + vs[b, :i + 1, h].sum(0)) / (P + i + 1)
                np.testing.assert_allclose(out[b, i, h], want, atol=1e-12)
    # (b) q = 0 -> uniform weights as well
    out0 = orc.attn(np.zeros_like(q), ks, vs, kp, vp, sl, 0.4, "f64")
    np.testing.assert_allclose(out0, out, atol=1e-12)
    # (c) constant V -> output is that constant whatever the scores
    c = rng.standard_normal(D)
    outc = orc.attn(q, ks, np.broadcast_to(c, vs.shape).copy(), kp,
                    np.broadcast_to(c, vp.shape).copy(), sl, 0.4, "f64")
    np.testing.assert_allclose(outc, np.broadcast_to(c, outc.shape), atol=1e-12)
    # (d) one prefix key aligned with q and made huge -> output tends to that key's V row
    kp_d = kp.copy()
    j = 3
    qd = np.ones_like(q)
    kp_d[j] = 1e3
    outd = orc.attn(qd, ks, vs, kp_d, vp, sl, 1.0, "f64")
    for h in range(Hq):
        np.testing.assert_allclose(outd[:, :, h], np.broadcast_to(vp[j, h], (B, S, D)), atol=1e-9)
    # (e) scale matters: scale 0 -> uniform
    outs = orc.attn(q, ks, vs, kp, vp, sl, 0.0, "f64")
    np.testing.assert_allclose(outs, out, atol=1e-12)


def test_padded_rows_never_reach_valid_outputs():
    rng = np.random.default_rng(9)
    B, P, S, Hq, Hkv, D = 5, 4, 6, 4, 1, 4
    q, ks, vs, kp, vp, sl = rand_problem(rng, B, P, S, Hq, Hkv, D)
    sl[:] = [6, 3, 0, 1, 5]
    clean = orc.attn(q, ks, vs, kp, vp, sl, 0.5, "f64")
    pad = np.arange(S)[None, :] >= sl[:, None]
    qn, ksn, vsn = q.copy(), ks.copy(), vs.copy()
    qn[pad] = np.nan
    ksn[pad] = np.nan
    vsn[pad] = np.nan
    poisoned = orc.attn(qn, ksn, vsn, kp, vp, sl, 0.5, "f64")
    assert not np.isnan(poisoned).any()
    assert np.array_equal(poisoned, clean)
    assert np.all(poisoned[pad] == 0.0)


def test_gqa_equals_mha_on_repeated_heads():
    """Query head h reads KV head h // G: expanding K/V by repeating each KV head G times in
    place and running as MHA gives the same result."""
    rng = np.random.default_rng(13)
    B, P, S, Hq, Hkv, D = 3, 5, 4, 6, 2, 4
    q, ks, vs, kp, vp, sl = rand_problem(rng, B, P, S, Hq, Hkv, D)
    G = Hq // Hkv
    out_g = orc.attn(q, ks, vs, kp, vp, sl, 0.5, "f64")
    out_m = orc.attn(q, np.repeat(ks, G, axis=2), np.repeat(vs, G, axis=2),
                     np.repeat(kp, G, axis=1), np.repeat(vp, G, axis=1), sl, 0.5, "f64")
    assert np.array_equal(out_g, out_m)
    # and distinct KV heads really are used by distinct query-head groups
    vs2 = vs.copy()
    vs2[:, :, 1] += 1.0
    out2 = orc.attn(q, ks, vs2, kp, vp, sl, 0.5, "f64")
    assert np.array_equal(out2[:, :, :G], out_g[:, :, :G])
    valid = np.arange(S)[None, :] < sl[:, None]
    assert np.all(np.abs(out2[:, :, G:] - out_g[:, :, G:])[valid] > 0)


def test_lse_matches_logsumexp_of_visible_scores():
    from scipy.special import logsumexp
    rng = np.random.default_rng(17)
    B, P, S, Hq, Hkv, D = 2, 8, 5, 2, 1, 4
    q, ks, vs, kp, vp, sl = rand_problem(rng, B, P, S, Hq, Hkv, D, ragged=False)
    out, lse = orc.attn(q, ks, vs, kp, vp, sl, 0.7, "f64", want_lse=True)
    for b in range(B):
        for h in range(Hq):
            for i in range(S):
                keys = np.concatenate([kp[:, 0], ks[b, :i + 1, 0]], axis=0)
                ref = logsumexp(0.7 * keys @ q[b, i, h])
                assert abs(lse[b, h, i] - ref) < 1e-12


def test_split_merge_identity():
    """Attention over prefix U suffix equals the log-sum-exp weighted merge of attention over
    each part (the identity the GPU's online-softmax combine relies on); checked through the
    oracle by running P=0 and suffix-free variants."""
    rng = np.random.default_rng(19)
    B, P, S, Hq, Hkv, D = 2, 6, 4, 2, 2, 4
    q, ks, vs, kp, vp, sl = rand_problem(rng, B, P, S, Hq, Hkv, D, ragged=False)
    full, lse_full = orc.attn(q, ks, vs, kp, vp, sl, 0.5, "f64", want_lse=True)
    suf, lse_suf = orc.attn(q, ks, vs, kp[:0], vp[:0], sl, 0.5, "f64", want_lse=True)
    # prefix-only attention for every query: treat each query as a one-token candidate whose
    # own key is pushed to -inf weight by a huge negative score
    pre = np.zeros_like(full)
    lse_pre = np.zeros_like(lse_full)
    for b in range(B):
        for i in range(S):
            for h in range(Hq):
                s = 0.5 * kp[:, h] @ q[b, i, h]
                m = s.max()
                e = np.exp(s - m)
                pre[b, i, h] = (e / e.sum()) @ vp[:, h]
                lse_pre[b, h, i] = m + np.log(e.sum())
    w_pre = np.exp(lse_pre - lse_full).transpose(0, 2, 1)[..., None]
    w_suf = np.exp(lse_suf - lse_full).transpose(0, 2, 1)[..., None]
    np.testing.assert_allclose(w_pre * pre + w_suf * suf, full, atol=1e-12)


def test_dtype_widening_is_exact():
    w = gen.custom_workload("t", 3, 5, 4, 1, 4, 4, 2, 8, "bf16")
    inp = gen.make_inputs(w, pad="nan")
    out_b = orc.attn(inp.q, inp.k_suf, inp.v_suf, inp.k_pre, inp.v_pre, inp.suf_len, inp.scale, "bf16")
    f = [inp.as_f32(n) for n in ("q", "k_suf", "v_suf", "k_pre", "v_pre")]
    out_f = orc.attn(*f, inp.suf_len, inp.scale, "f32")
    out_d = orc.attn(*[a.astype(np.float64) for a in f], inp.suf_len, inp.scale, "f64")
    assert np.array_equal(out_b, out_f) and np.array_equal(out_f, out_d)
    assert not np.isnan(out_b).any()


def test_flop_counter_against_counting():
    sl = np.array([3, 0, 5], dtype=np.int32)
    P, Hq, D = 4, 2, 8
    macs = 0
    for l in sl:
        for i in range(l):
            macs += (P + i + 1) * D * 2       # one score and one weighted V row per visible key
    assert orc.alg_flops(sl, P, Hq, D) == 2 * macs * Hq
    # App. B.1: per candidate ~ L_dec (2 N_p + L_dec) score/value pairs, up to the diagonal
    l, Np = 20, 128
    assert orc.alg_flops(np.array([l]), Np, 1, 1) == 2 * l * (2 * Np + l + 1)


def test_c_and_numpy_oracles_agree_on_config0():
    inp = gen.make_inputs(gen.WORKLOADS["tiny_f32"], pad="nan")
    a, la = orc.attn(inp.q, inp.k_suf, inp.v_suf, inp.k_pre, inp.v_pre, inp.suf_len, inp.scale,
                     "f32", want_lse=True)
    b, lb = orc.attn_numpy(inp.q, inp.k_suf, inp.v_suf, inp.k_pre, inp.v_pre, inp.suf_len,
                           inp.scale, "f32")
    np.testing.assert_allclose(a, b, atol=1e-13)
    v = np.isfinite(lb)
    np.testing.assert_allclose(la[v], lb[v], atol=1e-13)
    assert not np.isnan(a).any()
