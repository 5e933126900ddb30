"""GPU parity on seeded random shapes: prefix lengths on both sides of the resident/streamed
boundary and of the tile size, suffix-side segments of one to three key tiles, query-head groups
of 1 to 8 including 7, ragged lengths with empty candidates.  Forward through whatever kernel the
library picks, every second case also through the backward pass.  The shapes are drawn from a
fixed seed, so a failure names a reproducible case."""
import numpy as np
import pytest

from paper_2603_13420_amd import inputs as gen
import parity_util as pu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pk():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2603_13420_amd import binding
    binding.load()
    return binding


def draw_shape(case: int):
    rng = np.random.default_rng(977 + case)
    G = int(rng.choice([1, 2, 4, 7, 8]))
    Hkv = int(rng.choice([1, 2, 4]))
    P = int(rng.choice([0, rng.integers(1, 96), rng.integers(96, 257), rng.integers(257, 700)]))
    S = int(rng.choice([rng.integers(1, 33), rng.integers(33, 97), 8 * rng.integers(1, 13)]))
    B = int(rng.integers(1, 7))
    lo = int(rng.integers(0, S + 1))
    return B, P, S, lo, S, G * Hkv, Hkv


@pytest.mark.parametrize("case", range(32))
def test_random_shape(pk, case):
    import torch
    B, P, S, lo, hi, Hq, Hkv = draw_shape(case)
    w = gen.custom_workload(f"rand{case}", B, P, S, lo, hi, Hq, Hkv, 128, "bf16", index=1200 + case)
    inp = gen.make_inputs(w, pad="nan")
    d = pu.to_device(inp)
    print(f"[case] random shape {case}: B={B} P={P} S={S} len={lo}..{hi} Hq={Hq} Hkv={Hkv} seed={w.seed}", flush=True)
    lse = torch.full((B, Hq, S), 123.0, device="cuda:0")
    out = torch.full_like(d["q"], float("nan"))
    pk.pskv_attn_fwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], out=out, lse=lse,
                     scale=inp.scale)
    torch.cuda.synchronize()
    ref, ref_lse = pu.oracle_out(inp, want_lse=True)
    pu.compare_lse(lse.cpu().numpy().astype(np.float64), ref_lse, inp.suf_len, "bf16", w.name)
    print("      ", pu.compare(pu.out_to_f64(out), ref, inp.suf_len, "bf16", w.name), flush=True)
    if case % 2:
        return
    dout_host, dout64 = pu.make_dout(inp, w.seed + 7)
    dout = torch.from_numpy(dout_host).view(torch.bfloat16).to("cuda:0")
    dq, dk, dv = pk.pskv_attn_bwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], out, lse, dout,
                                  scale=inp.scale)
    torch.cuda.synchronize()
    # the oracle differentiates the exact forward pass; the kernels are handed the rounded `out`
    rq, rk, rv = pu.oracle_bwd(inp, dout64)
    valid = np.arange(S)[None, :] < inp.suf_len[:, None]
    for name, got, r in (("dq", dq, rq), ("dk_suf", dk, rk), ("dv_suf", dv, rv)):
        print("      ", name, pu.compare_grad(pu.out_to_f64(got), r, valid, "bf16", f"{w.name} {name}"), flush=True)


def draw_long_suffix_shape(case: int):
    """Suffix-side segments of four to seven key tiles (suffix, template tail and target together):
    the shapes that take the passes cut out of one candidate, or the streamed kernels' multi-step
    suffix, depending on the query-head group."""
    rng = np.random.default_rng(2977 + case)
    G = int(rng.choice([1, 2, 4, 7, 8]))
    Hkv = int(rng.choice([1, 2, 4]))
    P = int(rng.choice([0, rng.integers(1, 96), rng.integers(96, 257), rng.integers(257, 900)]))
    S = int(rng.choice([8 * rng.integers(13, 26), 32 * rng.integers(3, 7)]))
    B = int(rng.integers(1, 10))
    lo = int(rng.integers(0, S + 1))
    return B, P, S, lo, S, G * Hkv, Hkv


@pytest.mark.parametrize("case", range(12))
def test_random_long_suffix_shape(pk, case):
    import torch
    B, P, S, lo, hi, Hq, Hkv = draw_long_suffix_shape(case)
    w = gen.custom_workload(f"randlong{case}", B, P, S, lo, hi, Hq, Hkv, 128, "bf16", index=1400 + case)
    inp = gen.make_inputs(w, pad="nan")
    d = pu.to_device(inp)
    print(f"[case] random long-suffix shape {case}: B={B} P={P} S={S} len={lo}..{hi} Hq={Hq} Hkv={Hkv} seed={w.seed}", flush=True)
    lse = torch.full((B, Hq, S), 123.0, device="cuda:0")
    out = torch.full_like(d["q"], float("nan"))
    pk.pskv_attn_fwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], out=out, lse=lse,
                     scale=inp.scale)
    torch.cuda.synchronize()
    ref, ref_lse = pu.oracle_out(inp, want_lse=True)
    pu.compare_lse(lse.cpu().numpy().astype(np.float64), ref_lse, inp.suf_len, "bf16", w.name)
    print("      ", pu.compare(pu.out_to_f64(out), ref, inp.suf_len, "bf16", w.name), flush=True)
    dout_host, dout64 = pu.make_dout(inp, w.seed + 7)
    dout = torch.from_numpy(dout_host).view(torch.bfloat16).to("cuda:0")
    dq, dk, dv = pk.pskv_attn_bwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], out, lse, dout,
                                  scale=inp.scale)
    torch.cuda.synchronize()
    rq, rk, rv = pu.oracle_bwd(inp, dout64)
    valid = np.arange(S)[None, :] < inp.suf_len[:, None]
    for name, got, r in (("dq", dq, rq), ("dk_suf", dk, rk), ("dv_suf", dv, rv)):
        print("      ", name, pu.compare_grad(pu.out_to_f64(got), r, valid, "bf16", f"{w.name} {name}"), flush=True)


def draw_multi_shape(case: int):
    rng = np.random.default_rng(1977 + case)
    G = int(rng.choice([1, 2, 4, 7]))
    Hkv = int(rng.choice([1, 2, 4]))
    P = int(rng.choice([rng.integers(1, 96), rng.integers(96, 257), rng.integers(257, 600)]))
    plo = int(rng.integers(0, P + 1))
    S = int(rng.choice([rng.integers(1, 33), rng.integers(33, 80), 8 * rng.integers(1, 11)]))
    return int(rng.integers(1, 6)), int(rng.integers(1, 5)), P, plo, P, S, int(rng.integers(0, S + 1)), S, G * Hkv, Hkv


@pytest.mark.parametrize("case", range(12))
def test_random_multi_shape(pk, case):
    """The multi-instruction form on random shapes: prefixes of random real lengths (left-padded,
    padding NaN), forward through whatever kernel the library picks."""
    import torch
    Np, C, P, plo, phi, S, lo, hi, Hq, Hkv = draw_multi_shape(case)
    w = gen.custom_multi_workload(f"mrand{case}", Np, C, P, plo, phi, S, lo, hi, Hq, Hkv, 128, "bf16", index=1300 + case)
    inp = gen.make_multi_inputs(w, pad="nan")
    d = pu.to_device_multi(inp)
    print(f"[case] random multi shape {case}: Np={Np} C={C} P={P} pre_len={inp.pre_len.tolist()} S={S} len={lo}..{hi} "
          f"Hq={Hq} Hkv={Hkv} seed={w.seed}", flush=True)
    lse = torch.full((w.B, Hq, S), 123.0, device="cuda:0")
    out = torch.full_like(d["q"], float("nan"))
    pk.pskv_attn_fwd_multi(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["pre_len"], d["suf_len"],
                           out=out, lse=lse, scale=inp.scale)
    torch.cuda.synchronize()
    ref, ref_lse = pu.oracle_out_multi(inp, want_lse=True)
    pu.compare_lse(lse.cpu().numpy().astype(np.float64), ref_lse, inp.suf_len, "bf16", w.name)
    pu.compare(pu.out_to_f64(out), ref, inp.suf_len, "bf16", w.name)


@pytest.mark.parametrize("B,P,S,Hq,Hkv", [
    (3, 256, 24, 8, 2),     # resident prefix, pipelined kernel
    (2, 300, 32, 8, 2),     # streamed prefix
    (2, 130, 96, 8, 2),     # passes cut out of one candidate
    (2, 0, 1, 4, 4),        # no prefix, one-token suffixes
])
def test_degenerate_lengths(pk, B, P, S, Hq, Hkv):
    """All candidates empty (everything is padding: exact zeros, lse -inf, zero gradients), then all
    candidates one token long."""
    import torch
    for n in (0, 1):
        w = gen.custom_workload(f"degenerate_{P}_{S}_{n}", B, P, S, n, n, Hq, Hkv, 128, "bf16", index=1500 + P + n)
        inp = gen.make_inputs(w, pad="nan")
        d = pu.to_device(inp)
        print(f"[case] all lengths {n}: B={B} P={P} S={S} Hq={Hq} Hkv={Hkv} seed={w.seed}", flush=True)
        lse = torch.full((B, Hq, S), 123.0, device="cuda:0")
        out = torch.full_like(d["q"], float("nan"))
        pk.pskv_attn_fwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], out=out, lse=lse,
                         scale=inp.scale)
        torch.cuda.synchronize()
        ref, ref_lse = pu.oracle_out(inp, want_lse=True)
        pu.compare_lse(lse.cpu().numpy().astype(np.float64), ref_lse, inp.suf_len, "bf16", w.name)
        pu.compare(pu.out_to_f64(out), ref, inp.suf_len, "bf16", w.name)
        dout_host, dout64 = pu.make_dout(inp, w.seed + 7)
        dout = torch.from_numpy(dout_host).view(torch.bfloat16).to("cuda:0")
        dq, dk, dv = pk.pskv_attn_bwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], out, lse, dout,
                                      scale=inp.scale)
        torch.cuda.synchronize()
        rq, rk, rv = pu.oracle_bwd(inp, dout64)
        valid = np.arange(S)[None, :] < inp.suf_len[:, None]
        for name, got, r in (("dq", dq, rq), ("dk_suf", dk, rk), ("dv_suf", dv, rv)):
            pu.compare_grad(pu.out_to_f64(got), r, valid, "bf16", f"{w.name} {name}")
