"""GPU parity of the batched multi-instruction form (left-padded per-instruction prefixes,
C candidates per instruction): the HIP path through the C ABI against the CPU oracle on the
same seeded inputs.  Prefix padding rows and suffix padding rows are NaN-poisoned."""
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


def poison_padding(inp):
    """NaN into every prefix row before an instruction's real rows and every suffix row at or
    beyond a candidate's length (for inputs drawn with pad="keep" whose lengths were edited)."""
    w = inp.w
    nan = np.uint16(0x7FC0) if w.dtype == "bf16" else np.float32(np.nan)
    pre_pad = np.arange(w.P)[None, :] < (w.P - inp.pre_len)[:, None]
    inp.k_pre[pre_pad] = nan
    inp.v_pre[pre_pad] = nan
    suf_pad = np.arange(w.S)[None, :] >= inp.suf_len[:, None]
    for a in (inp.q, inp.k_suf, inp.v_suf):
        a[suf_pad] = nan
    return inp


def run_multi(pk, inp, impl, what=""):
    import torch
    d = pu.to_device_multi(inp)
    w = inp.w
    lse = torch.full((w.B, w.Hq, w.S), 123.0, device="cuda:0")
    out = torch.full_like(d["q"], float("nan"))
    print(f"[case] {what or w.name} impl={impl} Np={w.Np} C={w.C} P={w.P} pre_len={inp.pre_len.tolist()[:8]} "
          f"S={w.S} Hq={w.Hq} Hkv={w.Hkv} D={w.D} {w.dtype} seed={w.seed}", flush=True)
    pk.pskv_attn_fwd_multi(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["pre_len"], d["suf_len"],
                           out=out, lse=lse, impl=impl, scale=inp.scale)
    torch.cuda.synchronize()
    ref, ref_lse = pu.oracle_out_multi(inp, want_lse=True)
    pu.compare_lse(lse.cpu().numpy().astype(np.float64), ref_lse, inp.suf_len, w.dtype, what)
    res = pu.compare(pu.out_to_f64(out), ref, inp.suf_len, w.dtype, what or w.name)
    print(f"       {res}", flush=True)
    return res


@pytest.mark.parametrize("impl", ["simple", "mfma"])
@pytest.mark.parametrize("Np,C,P,plo,phi,S,lo,hi,Hq,Hkv", [
    (3, 4, 256, 96, 256, 24, 16, 24, 8, 2),     # resident prefixes, blocks inside one candidate
    (5, 2, 100, 0, 100, 20, 0, 20, 4, 4),       # several candidates per block, some prefixes empty or very short
    (4, 3, 160, 1, 160, 24, 1, 24, 8, 2),       # mix of pipelined (>= 3 tiles) and short prefixes in one launch
    (40, 1, 64, 10, 64, 16, 16, 16, 16, 8),     # 320 virtual heads: more than one per workgroup
    (3, 4, 700, 150, 700, 32, 5, 32, 8, 2),     # streamed prefixes, one suffix step; short ones take the general sweep
    (2, 3, 520, 300, 520, 64, 20, 64, 2, 2),    # streamed, two suffix steps
    (3, 2, 300, 0, 300, 33, 5, 33, 14, 2),      # streamed, general kernel (odd sizes, group 7)
    (4, 3, 200, 20, 200, 64, 1, 64, 8, 2),      # passes cut out of one candidate; short prefixes take the general sweep
])
def test_multi_small_shapes_bf16(pk, impl, Np, C, P, plo, phi, S, lo, hi, Hq, Hkv):
    w = gen.custom_multi_workload(f"multi_{Np}_{C}_{P}_{S}", Np, C, P, plo, phi, S, lo, hi, Hq, Hkv, 128, "bf16",
                                  index=300 + Np + P)
    inp = gen.make_multi_inputs(w, pad="keep")
    inp.pre_len[0] = phi                 # one instruction without any padding
    if plo == 0:
        inp.pre_len[-1] = 0              # and one without any prefix
    run_multi(pk, poison_padding(inp), impl)


def test_multi_f32(pk):
    w = gen.custom_multi_workload("multi_f32", 3, 3, 40, 0, 40, 12, 1, 12, 4, 2, 64, "f32", index=350)
    run_multi(pk, gen.make_multi_inputs(w, pad="nan"), "auto")


def test_single_instruction_call_equals_multi_with_one_instruction(pk):
    """pskv_attn_fwd and pskv_attn_fwd_multi(Np = 1, no pre_len) are the same operation: same bits."""
    import torch
    w = gen.custom_workload("one", 6, 256, 24, 16, 24, 8, 2, 128, "bf16", index=360)
    inp = gen.make_inputs(w, pad="nan")
    d = pu.to_device(inp)
    a = pk.pskv_attn_fwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], scale=inp.scale)
    b = pk.pskv_attn_fwd_multi(d["q"], d["k_suf"], d["v_suf"], d["k_pre"][None], d["v_pre"][None], None,
                               d["suf_len"], scale=inp.scale)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_strided_prefix_batch_and_clamped_prefix_lengths(pk):
    """Prefixes taken as a strided view of a larger buffer; pre_len values outside [0,P] are clamped."""
    import torch
    w = gen.custom_multi_workload("strided", 3, 2, 96, 20, 96, 16, 4, 16, 4, 2, 128, "bf16", index=361)
    inp = gen.make_multi_inputs(w, pad="keep")
    inp.pre_len[:] = [96, 0, 40]
    d = pu.to_device_multi(poison_padding(inp))
    big_k = torch.full((w.Np, w.P + 8, w.Hkv, w.D), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    big_v = torch.full_like(big_k, float("nan"))
    big_k[:, 8:] = d["k_pre"]
    big_v[:, 8:] = d["v_pre"]
    wild = torch.tensor([1000, -5, 40], dtype=torch.int32, device="cuda:0")
    out = pk.pskv_attn_fwd_multi(d["q"], d["k_suf"], d["v_suf"], big_k[:, 8:], big_v[:, 8:], wild, d["suf_len"],
                                 scale=inp.scale)
    torch.cuda.synchronize()
    ref = pu.oracle_out_multi(inp)
    pu.compare(pu.out_to_f64(out), ref, inp.suf_len, "bf16", "strided prefix batch")


@pytest.mark.parametrize("name", ["multi8_gqa8b_bf16", "multi32_gqa8b_bf16", "multi4_long_bf16"])
def test_multi_named_workloads_full_size(pk, name):
    """The multi-instruction workloads of the benchmark at full size, every element compared."""
    run_multi(pk, gen.make_multi_inputs(gen.MULTI_WORKLOADS[name], pad="nan"), "auto")


# ------------------------------------------------------------------------------------------
# backward pass of the multi-instruction form
# ------------------------------------------------------------------------------------------
def run_multi_bwd(pk, inp, impl, what=""):
    import torch
    d = pu.to_device_multi(inp)
    w = inp.w
    print(f"[case] bwd {what or w.name} impl={impl} Np={w.Np} C={w.C} P={w.P} pre_len={inp.pre_len.tolist()[:8]} "
          f"S={w.S} Hq={w.Hq} Hkv={w.Hkv} D={w.D} {w.dtype} seed={w.seed}", flush=True)
    lse = torch.empty((w.B, w.Hq, w.S), dtype=torch.float32, device="cuda:0")
    out = pk.pskv_attn_fwd_multi(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["pre_len"], d["suf_len"],
                                 lse=lse, scale=inp.scale)
    dout_host, dout64 = pu.make_dout(inp, w.seed + 7)
    t = torch.from_numpy(dout_host)
    dout = (t.view(torch.bfloat16) if w.dtype == "bf16" else t).to("cuda:0")
    nan = float("nan")
    dq, dk, dv = (torch.full_like(d["q"], nan), torch.full_like(d["k_suf"], nan), torch.full_like(d["k_suf"], nan))
    pk.pskv_attn_bwd_multi(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["pre_len"], d["suf_len"], out, lse,
                           dout, dq=dq, dk_suf=dk, dv_suf=dv, impl=impl, scale=inp.scale)
    torch.cuda.synchronize()
    rq, rk, rv = pu.oracle_bwd_multi(inp, dout64)   # exact gradients with their element-wise error bounds
    valid = np.arange(w.S)[None, :] < inp.suf_len[:, None]
    res = {n: pu.compare_grad(pu.out_to_f64(g), r, valid, w.dtype, f"{what or w.name} {n}")
           for n, g, r in (("dq", dq, rq), ("dk_suf", dk, rk), ("dv_suf", dv, rv))}
    print(f"       {res}", flush=True)
    return res


@pytest.mark.parametrize("impl", ["simple", "mfma"])
@pytest.mark.parametrize("Np,C,P,plo,phi,S,lo,hi,Hq,Hkv", [
    (3, 4, 256, 96, 256, 24, 16, 24, 8, 2),     # the headline shape in small, three instructions
    (5, 2, 100, 0, 100, 20, 0, 20, 4, 4),       # several candidates per block, some prefixes empty or very short
    (3, 2, 300, 0, 300, 33, 5, 33, 14, 2),      # group 7, odd sizes
    (2, 3, 520, 300, 520, 64, 20, 64, 2, 2),    # longer prefixes and suffix-side segments
])
def test_multi_bwd_small_shapes_bf16(pk, impl, Np, C, P, plo, phi, S, lo, hi, Hq, Hkv):
    w = gen.custom_multi_workload(f"multi_bwd_{Np}_{C}_{P}_{S}", Np, C, P, plo, phi, S, lo, hi, Hq, Hkv, 128, "bf16",
                                  index=400 + Np + P)
    inp = gen.make_multi_inputs(w, pad="keep")
    inp.pre_len[0] = phi
    if plo == 0:
        inp.pre_len[-1] = 0
    run_multi_bwd(pk, poison_padding(inp), impl)


def test_multi_bwd_f32(pk):
    w = gen.custom_multi_workload("multi_bwd_f32", 3, 3, 40, 0, 40, 12, 1, 12, 4, 2, 64, "f32", index=450)
    run_multi_bwd(pk, gen.make_multi_inputs(w, pad="nan"), "auto")


def test_single_instruction_backward_equals_multi_with_one_instruction(pk):
    """pskv_attn_bwd and pskv_attn_bwd_multi(Np = 1, no pre_len) are the same operation: same bits."""
    import torch
    w = gen.custom_workload("one_bwd", 6, 256, 24, 16, 24, 8, 2, 128, "bf16", index=460)
    inp = gen.make_inputs(w, pad="nan")
    d = pu.to_device(inp)
    lse = torch.empty((w.B, w.Hq, w.S), dtype=torch.float32, device="cuda:0")
    out = pk.pskv_attn_fwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], lse=lse, scale=inp.scale)
    dout_host, _ = pu.make_dout(inp, 461)
    dout = torch.from_numpy(dout_host).view(torch.bfloat16).to("cuda:0")
    a = pk.pskv_attn_bwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], out, lse, dout,
                         scale=inp.scale)
    b = pk.pskv_attn_bwd_multi(d["q"], d["k_suf"], d["v_suf"], d["k_pre"][None], d["v_pre"][None], None, d["suf_len"],
                               out, lse, dout, scale=inp.scale)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x.view(torch.int16), y.view(torch.int16))
