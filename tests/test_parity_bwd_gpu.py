"""GPU parity of the backward pass (gradients with respect to q, k_suf, v_suf; the prefix is a
constant) through the C ABI against the CPU oracle's backward on the same seeded inputs.  The
forward results the backward call consumes (out, lse) come from the HIP forward call, as they
would in use; padded rows of every input, dout included, are NaN-poisoned."""
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


make_dout, compare_grad = pu.make_dout, pu.compare_grad


def run_bwd(pk, inp, impl="auto", what=""):
    import torch
    w = inp.w
    d = pu.to_device(inp)
    print(f"[case] bwd {what or w.name} impl={impl} B={w.B} P={w.P} S={w.S} Hq={w.Hq} Hkv={w.Hkv} D={w.D} "
          f"{w.dtype} seed={w.seed}", flush=True)
    lse = torch.empty((w.B, w.Hq, w.S), dtype=torch.float32, device="cuda:0")
    out = pk.pskv_attn_fwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], lse=lse,
                           scale=inp.scale)
    dout_host, dout64 = make_dout(inp, w.seed + 7)
    t = torch.from_numpy(dout_host)
    dout = (t.view(torch.bfloat16) if w.dtype == "bf16" else t).to("cuda:0")
    nan = float("nan")
    dq, dk, dv = (torch.full_like(d["q"], nan), torch.full_like(d["k_suf"], nan), torch.full_like(d["k_suf"], nan))
    pk.pskv_attn_bwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], out, lse, dout,
                     dq=dq, dk_suf=dk, dv_suf=dv, impl=impl, scale=inp.scale)
    torch.cuda.synchronize()
    rq, rk, rv = pu.oracle_bwd(inp, dout64)     # exact gradients with their element-wise error bounds
    valid = np.arange(w.S)[None, :] < inp.suf_len[:, None]
    res = {n: compare_grad(pu.out_to_f64(g), r, valid, w.dtype, f"{what or w.name} {n}")
           for n, g, r in (("dq", dq, rq), ("dk_suf", dk, rk), ("dv_suf", dv, rv))}
    print(f"       {res}", flush=True)
    return res


def test_bwd_tiny_f32(pk):
    run_bwd(pk, gen.make_inputs(gen.WORKLOADS["tiny_f32"], pad="nan"))


@pytest.mark.parametrize("impl", ["simple", "mfma"])
@pytest.mark.parametrize("B,P,S,lo,hi,Hq,Hkv", [
    (5, 48, 16, 1, 16, 4, 4),       # MHA, ragged
    (6, 256, 24, 16, 24, 8, 2),     # GQA group 4, the headline shape in small
    (3, 0, 24, 0, 24, 4, 1),        # no prefix; one candidate may be empty
    (3, 300, 33, 5, 33, 14, 2),     # group 7, odd sizes, long prefix
    (2, 700, 70, 33, 70, 2, 2),     # long suffix-side segment
    (3, 128, 160, 100, 160, 8, 2),  # the scoring workload in small: resident prefix, five suffix steps
    (2, 100, 96, 40, 96, 14, 2),    # the same with a query-head group of 7 and a ragged prefix tile
    (3, 128, 160, 0, 160, 4, 1),    # passes cut out of one candidate: empty, short and full candidates
    (3, 300, 40, 5, 40, 8, 2),      # ... one pass of 5 blocks per unit, streamed prefix
    (9, 70, 64, 64, 64, 4, 1),      # ... more units than eight
    (2, 0, 96, 1, 96, 4, 2),        # ... no prefix at all
])
def test_bwd_small_shapes_bf16(pk, impl, B, P, S, lo, hi, Hq, Hkv):
    w = gen.custom_workload(f"bwd_{B}_{P}_{S}_{Hq}_{Hkv}", B, P, S, lo, hi, Hq, Hkv, 128, "bf16", index=800 + B + P)
    run_bwd(pk, gen.make_inputs(w, pad="nan"), impl=impl)


def test_bwd_headline_shape_sampled(pk):
    """The 8B-class GQA shape at full size through the matrix-core path; the oracle recomputes a
    sample of candidates (a candidate's gradients depend only on the prefix and on itself)."""
    import torch
    inp = gen.make_inputs(gen.WORKLOADS["gqa8b_bf16"], pad="nan", workers=16)
    w = inp.w
    d = pu.to_device(inp)
    lse = torch.empty((w.B, w.Hq, w.S), dtype=torch.float32, device="cuda:0")
    out = pk.pskv_attn_fwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], lse=lse, scale=inp.scale)
    dout_host, dout64 = make_dout(inp, w.seed + 7)
    dout = torch.from_numpy(dout_host).view(torch.bfloat16).to("cuda:0")
    dq, dk, dv = pk.pskv_attn_bwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], out, lse, dout,
                                  scale=inp.scale)
    torch.cuda.synchronize()
    cand = np.array(sorted({0, 1, w.B // 2, w.B - 1, int(np.argmin(inp.suf_len)), int(np.argmax(inp.suf_len))}))
    sub = inp.take(cand)
    rq, rk, rv = pu.oracle_bwd(sub, dout64[cand])
    sel = torch.from_numpy(cand).to("cuda:0")
    valid = np.arange(w.S)[None, :] < sub.suf_len[:, None]
    for n, gt, r in (("dq", dq, rq), ("dk_suf", dk, rk), ("dv_suf", dv, rv)):
        print("      ", n, compare_grad(pu.out_to_f64(gt[sel]), r, valid, "bf16", f"gqa8b {n}"), flush=True)
    pad = ~(torch.arange(w.S, device="cuda:0")[None, :] < d["suf_len"][:, None])
    assert (dq[pad] == 0).all() and (dk[pad] == 0).all() and (dv[pad] == 0).all()
    assert torch.isfinite(dq.float()).all() and torch.isfinite(dk.float()).all() and torch.isfinite(dv.float()).all()


@pytest.mark.parametrize("D", [32, 64, 256])
def test_bwd_other_head_dims(pk, D):
    for dtype in ("f32", "bf16"):
        w = gen.custom_workload(f"bwd_d{D}_{dtype}", 3, 21, 9, 0, 9, 6, 3, D, dtype, index=850 + D)
        run_bwd(pk, gen.make_inputs(w, pad="nan"))


def test_bwd_refuses_missing_lse_wrong_path_and_aliases(pk):
    import torch
    w = gen.custom_workload("bwd_err", 2, 16, 8, 8, 8, 2, 2, 128, "bf16", index=870)
    inp = gen.make_inputs(w, pad="zero")
    d = pu.to_device(inp)
    lse = torch.empty((w.B, w.Hq, w.S), dtype=torch.float32, device="cuda:0")
    out = pk.pskv_attn_fwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], lse=lse)
    with pytest.raises(ValueError):
        pk.pskv_attn_bwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], out, None, out)
    w32 = gen.custom_workload("bwd_err32", 2, 16, 8, 8, 8, 2, 2, 64, "f32", index=871)
    d32 = pu.to_device(gen.make_inputs(w32, pad="zero"))
    lse32 = torch.empty((2, 2, 8), dtype=torch.float32, device="cuda:0")
    out32 = pk.pskv_attn_fwd(d32["q"], d32["k_suf"], d32["v_suf"], d32["k_pre"], d32["v_pre"], d32["suf_len"], lse=lse32)
    with pytest.raises(pk.PskvError) as e:   # the matrix-core path is for bf16, D == 128
        pk.pskv_attn_bwd(d32["q"], d32["k_suf"], d32["v_suf"], d32["k_pre"], d32["v_pre"], d32["suf_len"], out32, lse32,
                         torch.ones_like(out32), impl="mfma")
    assert e.value.status == pk.PSKV_ERR_UNSUPPORTED
    with pytest.raises(pk.PskvError) as e:   # an output aliasing an input
        pk.pskv_attn_bwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], out, lse,
                         torch.ones_like(out), dq=d["q"])
    assert e.value.status == pk.PSKV_ERR_INVALID_ARG


def test_bwd_without_workspace_gives_the_same_bits(pk):
    """The scratch tensor only saves a second read of out: with and without it the gradients
    are the same bits (the same sum <dout,out> is formed in the same order either way)."""
    import torch
    w = gen.custom_workload("bwd_ws", 6, 256, 24, 16, 24, 8, 2, 128, "bf16", index=870)
    inp = gen.make_inputs(w, pad="nan")
    d = pu.to_device(inp)
    lse = torch.empty((w.B, w.Hq, w.S), dtype=torch.float32, device="cuda:0")
    out = pk.pskv_attn_fwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], lse=lse, scale=inp.scale)
    dout_host, _ = make_dout(inp, 871)
    dout = torch.from_numpy(dout_host).view(torch.bfloat16).to("cuda:0")
    args = (d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], out, lse, dout)
    with_ws = pk.pskv_attn_bwd(*args, scale=inp.scale)
    small = torch.empty(16, dtype=torch.uint8, device="cuda:0")     # too small: ignored
    without = pk.pskv_attn_bwd(*args, scale=inp.scale, workspace=False)
    too_small = pk.pskv_attn_bwd(*args, scale=inp.scale, workspace=small)
    torch.cuda.synchronize()
    for x, y, z in zip(with_ws, without, too_small):
        assert torch.equal(x.view(torch.int16), y.view(torch.int16))
        assert torch.equal(x.view(torch.int16), z.view(torch.int16))


@pytest.mark.parametrize("impl", ["simple", "mfma"])
@pytest.mark.parametrize("B,P,S,lo,hi", [
    (6, 256, 24, 16, 24),       # resident-prefix dq kernel (32-bit row offsets within a candidate)
    (3, 300, 33, 5, 33),        # streamed dq kernel, odd sizes
])
def test_bwd_strided_views_of_fused_buffers(pk, impl, B, P, S, lo, hi):
    """q, k, v (and their gradients) as column slices of [B,S,(Hq+2Hkv)*D] buffers, out and dout
    with a padded head stride: only strides change, the gradients must not."""
    import torch
    w = gen.custom_workload(f"bwd_strided_{P}_{S}", B, P, S, lo, hi, 8, 2, 128, "bf16", index=880)
    inp = gen.make_inputs(w, pad="nan")
    d = pu.to_device(inp)
    Hq, Hkv, D = w.Hq, w.Hkv, w.D
    nan = float("nan")
    fused = torch.full((B, S, Hq + 2 * Hkv, D), nan, dtype=torch.bfloat16, device="cuda:0")
    fused[:, :, :Hq] = d["q"]
    fused[:, :, Hq:Hq + Hkv] = d["k_suf"]
    fused[:, :, Hq + Hkv:] = d["v_suf"]
    q, ks, vs = fused[:, :, :Hq], fused[:, :, Hq:Hq + Hkv], fused[:, :, Hq + Hkv:]
    grads = torch.full_like(fused, nan)
    dq, dk, dv = grads[:, :, :Hq], grads[:, :, Hq:Hq + Hkv], grads[:, :, Hq + Hkv:]
    obuf = torch.full((B, S, Hq, 2 * D), nan, dtype=torch.bfloat16, device="cuda:0")
    out = obuf[..., :D]
    lse = torch.empty((B, Hq, S), dtype=torch.float32, device="cuda:0")
    pk.pskv_attn_fwd(q, ks, vs, d["k_pre"], d["v_pre"], d["suf_len"], out=out, lse=lse, scale=inp.scale)
    dout_host, dout64 = make_dout(inp, 881)
    dbuf = torch.full_like(obuf, nan)
    dbuf[..., :D] = torch.from_numpy(dout_host).view(torch.bfloat16).to("cuda:0")
    dout = dbuf[..., :D]
    pk.pskv_attn_bwd(q, ks, vs, d["k_pre"], d["v_pre"], d["suf_len"], out, lse, dout, dq=dq, dk_suf=dk, dv_suf=dv,
                     impl=impl, scale=inp.scale)
    torch.cuda.synchronize()
    rq, rk, rv = pu.oracle_bwd(inp, dout64)
    valid = np.arange(S)[None, :] < inp.suf_len[:, None]
    for n, g, r in (("dq", dq, rq), ("dk_suf", dk, rk), ("dv_suf", dv, rv)):
        compare_grad(pu.out_to_f64(g.contiguous()), r, valid, "bf16", f"strided {n}")
