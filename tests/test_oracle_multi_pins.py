"""Pins for the batched multi-instruction oracle (Sec. 4.3 suffix-centric alignment, App. F.1
padding): what the paper's definition and the mathematics fix, none of it through the HIP path.

A slip in the instruction map (b // C), in the left-padding offset, in the exclusion of padding
rows, or in the column bookkeeping of the probabilities fails at least one of these.
"""
import math

import numpy as np
import pytest
import torch

from oracle import pskv_oracle as orc


def rand_multi(rng, Np, C, Pp, S, Hq, Hkv, D, full_prefix=False):
    B = Np * C
    q = rng.standard_normal((B, S, Hq, D))
    ks = rng.standard_normal((B, S, Hkv, D))
    vs = rng.standard_normal((B, S, Hkv, D))
    kp = rng.standard_normal((Np, Pp, Hkv, D))
    vp = rng.standard_normal((Np, Pp, Hkv, D))
    pl = (np.full(Np, Pp) if full_prefix else rng.integers(0, Pp + 1, size=Np)).astype(np.int32)
    sl = rng.integers(0, S + 1, size=B).astype(np.int32)
    return q, ks, vs, kp, vp, pl, sl


def brute_force_multi(q, ks, vs, kp, vp, pl, sl, scale):
    """Independent scalar implementation: a visibility predicate over padded indices instead of
    copying and compacting, exact summation, head loop outermost."""
    B, S, Hq, D = q.shape
    Np, Pp, Hkv, _ = kp.shape
    C = B // Np
    G = Hq // Hkv
    out = np.zeros((B, S, Hq, D))
    lse = np.full((B, Hq, S), -np.inf)
    for h in range(Hq):
        kv = h // G
        for b in range(B):
            n = b // C
            for i in range(int(sl[b])):
                keys = [("p", j) for j in range(Pp) if j >= Pp - int(pl[n])] + [("s", t) for t in range(i + 1)]
                krow = lambda kind, j: kp[n, j, kv] if kind == "p" else ks[b, j, kv]
                vrow = lambda kind, j: vp[n, j, kv] if kind == "p" else vs[b, j, kv]
                sc = [scale * math.fsum(q[b, i, h, d] * krow(*key)[d] for d in range(D)) for key in keys]
                mx = max(sc)
                w = [math.exp(x - mx) for x in sc]
                z = math.fsum(w)
                for d in range(D):
                    out[b, i, h, d] = math.fsum(wi * vrow(*key)[d] for wi, key in zip(w, keys)) / z
                lse[b, h, i] = mx + math.log(z)
    return out, lse


@pytest.mark.parametrize("Np,C,Pp,S,Hq,Hkv,D", [(2, 2, 5, 3, 2, 1, 4), (3, 1, 4, 2, 2, 2, 3), (1, 3, 6, 2, 3, 1, 2),
                                                (2, 3, 3, 4, 4, 2, 3)])
def test_brute_force_on_tiny_inputs(Np, C, Pp, S, Hq, Hkv, D):
    rng = np.random.default_rng(100 + Np * 7 + C)
    q, ks, vs, kp, vp, pl, sl = rand_multi(rng, Np, C, Pp, S, Hq, Hkv, D)
    sl[0] = S
    scale = 1.0 / math.sqrt(D)
    out, lse = orc.attn_multi(q, ks, vs, kp, vp, pl, sl, scale, "f64", want_lse=True)
    ref, ref_lse = brute_force_multi(q, ks, vs, kp, vp, pl, sl, scale)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)
    valid = np.arange(S)[None, None, :] < sl[:, None, None]
    np.testing.assert_allclose(lse[np.broadcast_to(valid, lse.shape)], ref_lse[np.broadcast_to(valid, lse.shape)],
                               rtol=0, atol=1e-12)


def test_one_candidate_per_instruction_is_masked_library_attention():
    """C = 1: each sequence is [left-padded prefix ; suffix]; a library attention routine with
    the ordinary padding + causal mask must agree."""
    rng = np.random.default_rng(7)
    Np, Pp, S, Hq, Hkv, D = 4, 9, 6, 4, 2, 8
    q, ks, vs, kp, vp, pl, sl = rand_multi(rng, Np, 1, Pp, S, Hq, Hkv, D)
    pl[:] = [9, 4, 1, 6]
    sl[:] = [6, 3, 5, 1]
    scale = 1.0 / math.sqrt(D)
    out = orc.attn_multi(q, ks, vs, kp, vp, pl, sl, scale, "f64")
    G = Hq // Hkv
    for n in range(Np):
        K = torch.from_numpy(np.concatenate([kp[n], ks[n]], axis=0)).permute(1, 0, 2).repeat_interleave(G, dim=0)
        V = torch.from_numpy(np.concatenate([vp[n], vs[n]], axis=0)).permute(1, 0, 2).repeat_interleave(G, dim=0)
        Q = torch.from_numpy(q[n]).permute(1, 0, 2)                                      # [Hq, S, D]
        col = torch.arange(Pp + S)[None, :]
        row = torch.arange(S)[:, None]
        mask = ((col >= Pp - int(pl[n])) & (col < Pp)) | ((col >= Pp) & (col - Pp <= row))
        ref = torch.nn.functional.scaled_dot_product_attention(Q, K, V, attn_mask=mask[None], scale=scale)
        ref = ref.permute(1, 0, 2).numpy()
        L = int(sl[n])
        np.testing.assert_allclose(out[n, :L], ref[:L], rtol=0, atol=1e-12)
        assert (out[n, L:] == 0).all()


def test_single_instruction_without_padding_is_the_single_prefix_oracle():
    rng = np.random.default_rng(8)
    q, ks, vs, kp, vp, pl, sl = rand_multi(rng, 1, 5, 7, 4, 4, 2, 8, full_prefix=True)
    a = orc.attn_multi(q, ks, vs, kp, vp, pl, sl, 0.3, "f64")
    b = orc.attn(q, ks, vs, kp[0], vp[0], sl, 0.3, "f64")
    assert np.array_equal(a, b)
    c = orc.attn_multi(q, ks, vs, kp, vp, None, sl, 0.3, "f64")   # pre_len omitted: no padding
    assert np.array_equal(a, c)


def test_padding_rows_never_matter_and_padding_amount_is_irrelevant():
    """Poisoning the padding rows with NaN changes nothing, and padding every prefix further to
    the left (larger Pp, same real rows) gives bit-identical outputs."""
    rng = np.random.default_rng(9)
    Np, C, Pp, S, Hq, Hkv, D = 3, 2, 8, 5, 4, 2, 8
    q, ks, vs, kp, vp, pl, sl = rand_multi(rng, Np, C, Pp, S, Hq, Hkv, D)
    pl[:] = [8, 3, 0]
    base, probs = orc.attn_multi(q, ks, vs, kp, vp, pl, sl, 0.25, "f64", want_probs=True)
    kp2, vp2 = kp.copy(), vp.copy()
    for n in range(Np):
        kp2[n, :Pp - pl[n]] = np.nan
        vp2[n, :Pp - pl[n]] = np.nan
    poisoned = orc.attn_multi(q, ks, vs, kp2, vp2, pl, sl, 0.25, "f64")
    assert np.array_equal(base, poisoned) and np.isfinite(poisoned).all()
    extra = 5
    kp3 = np.concatenate([np.full((Np, extra, Hkv, D), np.nan), kp2], axis=1)
    vp3 = np.concatenate([np.full((Np, extra, Hkv, D), np.nan), vp2], axis=1)
    shifted = orc.attn_multi(q, ks, vs, kp3, vp3, pl, sl, 0.25, "f64")
    assert np.array_equal(base, shifted)
    # probabilities: zero on padding columns and on future suffix columns, rows sum to one
    B = Np * C
    for b in range(B):
        n = b // C
        assert (probs[b, :, :, :Pp - pl[n]] == 0).all()
        for i in range(int(sl[b])):
            assert (probs[b, :, i, Pp + i + 1:] == 0).all()
            np.testing.assert_allclose(probs[b, :, i].sum(-1), 1.0, rtol=0, atol=1e-12)


def test_instructions_are_independent_and_candidates_follow_their_instruction():
    """Swapping two instructions (with their candidates) swaps the outputs bit for bit; changing
    one instruction's prefix changes only its own candidates."""
    rng = np.random.default_rng(10)
    Np, C, Pp, S, Hq, Hkv, D = 3, 2, 6, 4, 2, 2, 4
    q, ks, vs, kp, vp, pl, sl = rand_multi(rng, Np, C, Pp, S, Hq, Hkv, D)
    pl[:] = [6, 2, 4]
    sl[:] = np.maximum(sl, 1)
    base = orc.attn_multi(q, ks, vs, kp, vp, pl, sl, 0.5, "f64")
    perm = np.array([2, 0, 1])
    cperm = (perm[:, None] * C + np.arange(C)[None, :]).reshape(-1)
    swapped = orc.attn_multi(q[cperm], ks[cperm], vs[cperm], kp[perm], vp[perm], pl[perm], sl[cperm], 0.5, "f64")
    assert np.array_equal(swapped, base[cperm])
    kp4 = kp.copy()
    kp4[1] += 1.0
    changed = orc.attn_multi(q, ks, vs, kp4, vp, pl, sl, 0.5, "f64")
    assert np.array_equal(changed[:C], base[:C]) and np.array_equal(changed[2 * C:], base[2 * C:])
    assert not np.array_equal(changed[C:2 * C], base[C:2 * C])


def test_closed_forms_with_padding():
    """All real keys equal: uniform weights over pre_len + i + 1 rows, so the output is the mean
    of the visible V rows; an instruction with an empty prefix is plain causal attention."""
    rng = np.random.default_rng(11)
    Np, C, Pp, S, Hq, Hkv, D = 2, 2, 5, 3, 2, 1, 4
    q, ks, vs, kp, vp, pl, sl = rand_multi(rng, Np, C, Pp, S, Hq, Hkv, D)
    pl[:] = [3, 0]
    sl[:] = S
    kp[:] = 0.7
    ks[:] = 0.7
    out = orc.attn_multi(q, ks, vs, kp, vp, pl, sl, 1.0, "f64")
    for b in range(Np * C):
        n = b // C
        for i in range(S):
            vis = np.concatenate([vp[n, Pp - pl[n]:, 0], vs[b, :i + 1, 0]], axis=0)
            np.testing.assert_allclose(out[b, i, 0], vis.mean(0), rtol=0, atol=1e-12)
    plain = orc.attn(q[C:], ks[C:], vs[C:], np.zeros((0, Hkv, D)), np.zeros((0, Hkv, D)), sl[C:], 1.0, "f64")
    assert np.array_equal(out[C:], plain)


def test_bf16_and_f32_inputs_are_widened_exactly():
    from paper_2603_13420_amd import inputs as gen
    rng = np.random.default_rng(12)
    q, ks, vs, kp, vp, pl, sl = rand_multi(rng, 2, 2, 4, 3, 2, 1, 8)
    bits = [gen.f32_to_bf16_bits(x.astype(np.float32)) for x in (q, ks, vs, kp, vp)]
    wide = [gen.bf16_bits_to_f32(b).astype(np.float64) for b in bits]
    a = orc.attn_multi(*bits, pl, sl, 0.35, "bf16")
    b = orc.attn_multi(*wide, pl, sl, 0.35, "f64")
    assert np.array_equal(a, b)
