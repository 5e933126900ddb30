"""GPU parity with tensors of more than 2^31 elements: the first and the last candidates sit on
either side of where a 32-bit element or byte offset would wrap.  The tensors are drawn on the
device (seeded; a host draw of this size would take minutes), the sampled candidates are copied
back and recomputed by the oracle one by one (a candidate depends only on the prefix and itself)."""
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


def draw_on_device(B, P, S, lo, hi, Hq, Hkv, D, seed):
    import torch
    g = torch.Generator(device="cuda:0")
    g.manual_seed(seed)
    mk = lambda *shape: torch.randn(*shape, generator=g, device="cuda:0", dtype=torch.float32).to(torch.bfloat16)
    d = {"k_pre": mk(P, Hkv, D), "v_pre": mk(P, Hkv, D)}
    for name, H in (("q", Hq), ("k_suf", Hkv), ("v_suf", Hkv)):
        t = torch.empty((B, S, H, D), device="cuda:0", dtype=torch.bfloat16)
        for b0 in range(0, B, 1024):     # in slabs: the fp32 draw of a whole tensor would double its footprint
            t[b0:b0 + 1024] = mk(min(1024, B - b0), S, H, D)
        d[name] = t
    d["suf_len"] = torch.randint(lo, hi + 1, (B,), generator=g, device="cuda:0", dtype=torch.int32)
    return d


def subset_inputs(d, cand, name, P, S, lo, hi, Hq, Hkv, D, scale):
    """Host-side gen.Inputs of the listed candidates (bf16 as uint16 bits, padding NaN)."""
    import torch
    idx = torch.from_numpy(cand).to("cuda:0")
    bits = lambda t: t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    w = gen.custom_workload(name, len(cand), P, S, lo, hi, Hq, Hkv, D, "bf16", index=0)
    return gen.Inputs(w, bits(d["q"][idx]), bits(d["k_suf"][idx]), bits(d["v_suf"][idx]), bits(d["k_pre"]),
                      bits(d["v_pre"]), d["suf_len"][idx].cpu().numpy().astype(np.int32), scale)


@pytest.mark.parametrize("B,P,S,lo,hi,Hq,Hkv,backward", [
    (22000, 256, 24, 16, 24, 32, 8, True),    # the headline shape, 2.16e9 query elements: resident kernels
    (9000, 300, 64, 32, 64, 40, 40, False),   # 2.95e9 query elements: streamed kernel, two suffix steps
])
def test_tensors_beyond_2_31_elements(pk, B, P, S, lo, hi, Hq, Hkv, backward):
    import torch
    D = 128
    assert B * S * Hq * D > 2 ** 31
    print(f"[case] huge B={B} P={P} S={S} len={lo}..{hi} Hq={Hq} Hkv={Hkv} backward={backward}", flush=True)
    d = draw_on_device(B, P, S, lo, hi, Hq, Hkv, D, seed=20261999 + B)
    scale = float(np.float32(1.0 / np.sqrt(D)))
    lse = torch.empty((B, Hq, S), device="cuda:0", dtype=torch.float32)
    out = torch.full_like(d["q"], float("nan"))
    pk.pskv_attn_fwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], out=out, lse=lse, scale=scale)
    torch.cuda.synchronize()
    valid = torch.arange(S, device="cuda:0")[None, :] < d["suf_len"][:, None]
    assert (out[~valid] == 0).all(), "padded rows must be exactly 0"
    assert torch.isfinite(out[valid].float()).all()
    cand = np.array([0, 1, B // 2, B - 2, B - 1], dtype=np.int64)
    sub = subset_inputs(d, cand, "huge_subset", P, S, lo, hi, Hq, Hkv, D, scale)
    idx = torch.from_numpy(cand).to("cuda:0")
    ref, ref_lse = pu.oracle_out(sub, want_lse=True)
    pu.compare_lse(lse[idx].cpu().numpy().astype(np.float64), ref_lse, sub.suf_len, "bf16", "huge")
    res = pu.compare(pu.out_to_f64(out[idx]), ref, sub.suf_len, "bf16", "huge")
    print(f"       forward, {len(cand)} candidates: {res}", flush=True)
    if not backward:
        return
    g = torch.Generator(device="cuda:0")
    g.manual_seed(7)
    dout = torch.empty_like(out)
    for b0 in range(0, B, 1024):
        dout[b0:b0 + 1024] = torch.randn((min(1024, B - b0), S, Hq, D), generator=g, device="cuda:0").to(torch.bfloat16)
    nan = float("nan")
    dq, dk, dv = torch.full_like(d["q"], nan), torch.full_like(d["k_suf"], nan), torch.full_like(d["k_suf"], nan)
    pk.pskv_attn_bwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], out, lse, dout,
                     dq=dq, dk_suf=dk, dv_suf=dv, scale=scale)
    torch.cuda.synchronize()
    for t in (dq, dk, dv):
        assert (t[~valid] == 0).all(), "padded rows of the gradients must be exactly 0"
    dout64 = dout[idx].float().cpu().numpy().astype(np.float64)
    rq, rk, rv = pu.oracle_bwd(sub, dout64)
    vs = np.arange(S)[None, :] < sub.suf_len[:, None]
    for name, got, r in (("dq", dq, rq), ("dk_suf", dk, rk), ("dv_suf", dv, rv)):
        res = pu.compare_grad(pu.out_to_f64(got[idx]), r, vs, "bf16", f"huge {name}")
        print(f"       backward {name}: {res}", flush=True)


@pytest.mark.parametrize("B,P,S,lo,hi,backward", [
    (3, 256, 24, 16, 24, True),     # would take the resident pipelined kernels
    (2, 300, 32, 20, 32, False),    # would take the streamed pipelined kernel
    (2, 130, 96, 60, 96, False),    # would take the candidate passes
])
def test_candidate_spans_beyond_2_31_bytes(pk, B, P, S, lo, hi, backward):
    """Views with a token stride so large that one candidate's part of q, out and the suffix K/V
    spans more than 2^31 bytes: the kernels that keep 32-bit offsets within a candidate must not be
    chosen (or must not wrap); the result is the one of the contiguous call."""
    import torch
    Hq, Hkv, D = 8, 2, 128
    w = gen.custom_workload(f"span_{P}_{S}", B, P, S, lo, hi, Hq, Hkv, D, "bf16", index=1400 + P)
    inp = gen.make_inputs(w, pad="nan")
    d = pu.to_device(inp)
    row = (2 ** 31) // (2 * (S - 1)) + 4096        # elements per token row of the wide buffers
    row -= row % 8                                  # keeps every row 16-byte aligned
    assert (S - 1) * row * 2 >= 2 ** 31
    print(f"[case] wide strides B={B} P={P} S={S} token stride {row} elements seed={w.seed}", flush=True)
    wide = lambda H: torch.zeros((B, S, row), dtype=torch.bfloat16, device="cuda:0")[:, :, :H * D].view(B, S, H, D)
    q, ks, vs, out = wide(Hq), wide(Hkv), wide(Hkv), wide(Hq)
    q.copy_(d["q"]); ks.copy_(d["k_suf"]); vs.copy_(d["v_suf"])
    out.fill_(float("nan"))
    lse = torch.empty((B, Hq, S), dtype=torch.float32, device="cuda:0")
    pk.pskv_attn_fwd(q, ks, vs, d["k_pre"], d["v_pre"], d["suf_len"], out=out, lse=lse, scale=inp.scale)
    torch.cuda.synchronize()
    res = pu.compare(pu.out_to_f64(out.contiguous()), pu.oracle_out(inp), inp.suf_len, "bf16", "wide strides")
    print(f"       {res}", flush=True)
    if not backward:
        return
    dout_host, dout64 = pu.make_dout(inp, w.seed + 7)
    dout, dq, dk, dv = wide(Hq), wide(Hq), wide(Hkv), wide(Hkv)
    dout.copy_(torch.from_numpy(dout_host).view(torch.bfloat16).to("cuda:0"))
    for t in (dq, dk, dv):
        t.fill_(float("nan"))
    pk.pskv_attn_bwd(q, ks, vs, d["k_pre"], d["v_pre"], d["suf_len"], out, lse, dout, dq=dq, dk_suf=dk, dv_suf=dv,
                     scale=inp.scale)
    torch.cuda.synchronize()
    rq, rk, rv = pu.oracle_bwd(inp, dout64)
    valid = np.arange(S)[None, :] < inp.suf_len[:, None]
    for name, got, r in (("dq", dq, rq), ("dk_suf", dk, rk), ("dv_suf", dv, rv)):
        pu.compare_grad(pu.out_to_f64(got.contiguous()), r, valid, "bf16", f"wide strides {name}")
