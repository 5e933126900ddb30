"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Padded rows are NaN-poisoned in every case."""
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
    binding.load()   # raises if the HIP library is missing: there is no fallback
    return binding


def run_case(pk, inp, impl, want_lse=True, what=""):
    import torch
    d = pu.to_device(inp)
    w = inp.w
    lse = torch.full((w.B, w.Hq, w.S), 123.0, device="cuda:0") if want_lse else None
    out = torch.full_like(d["q"], float("nan"))
    print(f"[case] {what or w.name} impl={impl} B={w.B} P={w.P} S={w.S} Hq={w.Hq} Hkv={w.Hkv} "
          f"D={w.D} {w.dtype} seed={w.seed}", flush=True)
    pk.pskv_attn_fwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"],
                     out=out, lse=lse, impl=impl, scale=inp.scale)
    torch.cuda.synchronize()
    got = pu.out_to_f64(out)
    if want_lse:
        ref, ref_lse = pu.oracle_out(inp, want_lse=True)
        pu.compare_lse(lse.cpu().numpy().astype(np.float64), ref_lse, inp.suf_len, w.dtype, what)
    else:
        ref = pu.oracle_out(inp)
    res = pu.compare(got, ref, inp.suf_len, w.dtype, what or w.name)
    print(f"       {res}", flush=True)
    return res


IMPLS_BF16 = ["simple", "mfma"]


def test_tiny_f32_full(pk):
    run_case(pk, gen.make_inputs(gen.WORKLOADS["tiny_f32"], pad="nan"), "auto")
    run_case(pk, gen.make_inputs(gen.WORKLOADS["tiny_f32"], pad="nan"), "simple")


@pytest.mark.parametrize("impl", IMPLS_BF16)
@pytest.mark.parametrize("B,P,S,lo,hi,Hq,Hkv", [
    (5, 48, 16, 1, 16, 4, 4),       # several row tiles of one candidate, ragged
    (7, 100, 20, 20, 20, 8, 8),     # MHA, S not a multiple of 16, P not a multiple of 64
    (6, 256, 24, 16, 24, 8, 2),     # GQA group 4, the headline shape in small
    (3, 0, 24, 0, 24, 4, 1),        # no prefix at all: plain causal attention per candidate
    (4, 17, 1, 0, 1, 4, 2),         # one-token suffixes, some empty
    (3, 300, 33, 5, 33, 14, 2),     # group 7 (28/4-style), odd sizes everywhere
    (2, 700, 70, 33, 70, 2, 2),     # suffix longer than one key tile
    (1, 64, 16, 16, 16, 1, 1),      # single candidate, single head
    (3, 300, 32, 5, 32, 8, 2),      # streamed prefix, blocks inside one candidate, one suffix step
    (9, 289, 32, 0, 32, 4, 1),      # ... ragged last prefix tile, last pass with idle wavefronts
    (3, 420, 64, 20, 64, 2, 2),     # ... two suffix steps, second row block sometimes all padding
    (2, 1000, 96, 1, 96, 3, 3),     # ... three suffix steps
    (3, 300, 40, 5, 40, 8, 2),      # passes cut out of one candidate: one pass of 5 blocks, 6 units of 8
    (2, 130, 160, 100, 160, 8, 2),  # ... 20 blocks in three passes, five suffix tiles
    (3, 128, 160, 0, 160, 4, 1),    # ... prefix of whole tiles; empty, short and full candidates
    (2, 97, 96, 1, 96, 14, 2),      # ... group 7: blocks straddle suffix tiles; one-row last prefix tile
    (9, 70, 64, 64, 64, 4, 1),      # ... more units than eight, shortest prefix the pipeline takes
])
def test_small_shapes_bf16(pk, impl, B, P, S, lo, hi, Hq, Hkv):
    w = gen.custom_workload(f"small_{B}_{P}_{S}_{Hq}_{Hkv}", B, P, S, lo, hi, Hq, Hkv, 128, "bf16",
                            index=200 + B + P)
    run_case(pk, gen.make_inputs(w, pad="nan"), impl)


@pytest.mark.parametrize("D", [32, 64, 256])
def test_other_head_dims_simple(pk, D):
    for dtype in ("f32", "bf16"):
        w = gen.custom_workload(f"d{D}_{dtype}", 3, 21, 9, 0, 9, 6, 3, D, dtype, index=300 + D)
        run_case(pk, gen.make_inputs(w, pad="nan"), "simple")


@pytest.mark.parametrize("impl", ["simple", "mfma"])
def test_suf_len_null_means_full_length(pk, impl):
    import torch
    w = gen.custom_workload("full", 4, 40, 12, 12, 12, 4, 2, 128, "bf16", index=400)
    inp = gen.make_inputs(w, pad="nan")
    d = pu.to_device(inp)
    out = pk.pskv_attn_fwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], None, impl=impl, scale=inp.scale)
    torch.cuda.synchronize()
    pu.compare(pu.out_to_f64(out), pu.oracle_out(inp), inp.suf_len, "bf16", "suf_len=NULL")


@pytest.mark.parametrize("impl", ["simple", "mfma"])
@pytest.mark.parametrize("B,P,S,lo,hi", [
    (5, 70, 18, 3, 18),         # general kernels
    (6, 256, 24, 16, 24),       # resident prefix, pipelined kernel (32-bit row offsets within a candidate)
    (3, 300, 32, 5, 32),        # streamed prefix, pipelined kernel
    (2, 130, 160, 100, 160),    # passes cut out of one candidate
])
def test_strided_views_of_a_fused_qkv_buffer(pk, impl, B, P, S, lo, hi):
    """q, k, v as column slices of one [B,S,(Hq+2Hkv)*D] projection output, out with a
    padded head stride: only strides change, the result must not."""
    import torch
    w = gen.custom_workload(f"strided_{P}_{S}", B, P, S, lo, hi, 8, 2, 128, "bf16", index=401)
    inp = gen.make_inputs(w, pad="nan")
    d = pu.to_device(inp)
    B, S, Hq, Hkv, D = w.B, w.S, w.Hq, w.Hkv, w.D
    fused = torch.full((B, S, Hq + 2 * Hkv, D), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    fused[:, :, :Hq] = d["q"]
    fused[:, :, Hq:Hq + Hkv] = d["k_suf"]
    fused[:, :, Hq + Hkv:] = d["v_suf"]
    kv_pre = torch.stack([d["k_pre"], d["v_pre"]], dim=2)       # [P,Hkv,2,D]
    out_buf = torch.full((B, S, Hq, 2 * D), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    out = out_buf[..., :D]
    pk.pskv_attn_fwd(fused[:, :, :Hq], fused[:, :, Hq:Hq + Hkv], fused[:, :, Hq + Hkv:],
                     kv_pre[:, :, 0], kv_pre[:, :, 1], d["suf_len"], out=out, impl=impl, scale=inp.scale)
    torch.cuda.synchronize()
    pu.compare(pu.out_to_f64(out.contiguous()), pu.oracle_out(inp), inp.suf_len, "bf16", "strided")
    assert torch.isnan(out_buf[..., D:]).all()      # nothing written outside the view


def test_out_of_range_lengths_are_clamped(pk):
    import torch
    w = gen.custom_workload("clamp", 4, 30, 8, 8, 8, 2, 2, 128, "bf16", index=402)
    inp = gen.make_inputs(w, pad="keep")
    d = pu.to_device(inp)
    weird = torch.tensor([-3, 8, 100, 0], dtype=torch.int32, device="cuda:0")
    clamped = np.array([0, 8, 8, 0], dtype=np.int32)
    ref = pu.oracle_out(gen.Inputs(inp.w, inp.q, inp.k_suf, inp.v_suf, inp.k_pre, inp.v_pre,
                                   clamped, inp.scale))
    for impl in ("simple", "mfma"):
        out = pk.pskv_attn_fwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], weird, impl=impl, scale=inp.scale)
        torch.cuda.synchronize()
        pu.compare(pu.out_to_f64(out), ref, clamped, "bf16", f"clamp {impl}")


def test_runs_on_a_side_stream_and_is_deterministic(pk):
    import torch
    w = gen.custom_workload("stream", 6, 128, 20, 20, 20, 8, 8, 128, "bf16", index=403)
    inp = gen.make_inputs(w, pad="nan")
    d = pu.to_device(inp)
    ref = pu.oracle_out(inp)
    side = torch.cuda.Stream()
    outs = []
    with torch.cuda.stream(side):
        for _ in range(2):
            outs.append(pk.pskv_attn_fwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"],
                                         d["suf_len"], impl="auto", scale=inp.scale))
    side.synchronize()
    assert torch.equal(outs[0].view(torch.uint16), outs[1].view(torch.uint16))
    pu.compare(pu.out_to_f64(outs[0]), ref, inp.suf_len, "bf16", "side stream")


BF16_ONE, BF16_EIGHT = 0x3F80, 0x4100


@pytest.mark.parametrize("impl", ["simple", "mfma"])
@pytest.mark.parametrize("B,P,S,lo,hi,Hq,Hkv", [
    (4, 256, 24, 16, 24, 8, 2),     # blocks inside one candidate, one suffix step: pipelined kernel
    (5, 100, 20, 20, 20, 4, 4),     # several candidates per block: general resident kernel
    (3, 700, 40, 33, 40, 2, 2),     # long prefix: general streaming kernel
    (3, 700, 32, 20, 32, 8, 2),     # long prefix: pipelined streaming kernel, one suffix step
    (3, 400, 64, 40, 64, 2, 2),     # ... several suffix steps
    (3, 200, 96, 70, 96, 8, 2),     # passes cut out of one candidate
])
def test_scores_far_above_the_first_tile(pk, impl, B, P, S, lo, hi, Hq, Hkv):
    """A late prefix key and a late suffix key whose scores exceed everything seen before by
    ~90 in natural units: any softmax that fixes its reference early must notice and recover
    (the plain definition, which the oracle follows, subtracts the true maximum)."""
    w = gen.custom_workload(f"spike_{B}_{P}_{S}", B, P, S, lo, hi, Hq, Hkv, 128, "bf16", index=600 + P)
    inp = gen.make_inputs(w, pad="nan")
    # candidate 1: all-ones queries against an all-eights prefix key near the end of the prefix
    inp.q[1, :inp.suf_len[1]] = BF16_ONE
    inp.k_pre[P - 3] = BF16_EIGHT
    # candidate 2: all-ones queries against an all-eights key at its own last suffix position
    inp.q[2, :inp.suf_len[2]] = BF16_ONE
    inp.k_suf[2, inp.suf_len[2] - 1] = BF16_EIGHT
    res = run_case(pk, inp, impl, what=f"spike {w.name}")
    assert res["n"] > 0


def test_mha7b_full_size_full_compare(pk):
    """7B-class MHA shape at its full size, every output element compared."""
    inp = gen.make_inputs(gen.WORKLOADS["mha7b_bf16"], pad="nan")
    run_case(pk, inp, "auto")


def test_gqa8b_full_size_full_compare(pk):
    """8B-class GQA shape (the benchmark's configuration) at full size, every element."""
    inp = gen.make_inputs(gen.WORKLOADS["gqa8b_bf16"], pad="nan")
    run_case(pk, inp, "auto")


@pytest.mark.parametrize("name,chunk", [("longprefix_bf16", 64), ("mha13b_bf16", 256),
                                        ("ldec_gqa8b_bf16", 64), ("ldec_qwen7b_bf16", 64)])
def test_large_shapes_full_size_full_compare(pk, name, chunk):
    """Run at full size in the benchmark's launch configuration and compare EVERY valid element: the
    oracle goes over the candidates in chunks (a candidate depends only on the prefix and itself), so
    that its double-precision tensors of the largest workload never exist all at once."""
    import torch
    inp = gen.make_inputs(gen.WORKLOADS[name], pad="nan", workers=16)
    w = inp.w
    print(f"[case] {name} full size, full compare in chunks of {chunk} candidates", flush=True)
    d = pu.to_device(inp)
    out = pk.pskv_attn_fwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], impl="auto",
                            scale=inp.scale)
    torch.cuda.synchronize()
    worst = {}
    n_el = 0
    for lo in range(0, w.B, chunk):
        cand = np.arange(lo, min(w.B, lo + chunk))
        sub = inp.take(cand)
        res = pu.compare(pu.out_to_f64(out[lo:lo + len(cand)]), pu.oracle_out(sub), sub.suf_len, "bf16",
                         f"{name} candidates {lo}..{lo + len(cand) - 1}")
        n_el += res["n"]
        for k in ("max_abs", "max_abs_over_std", "bound_ratio", "rms_ratio"):
            worst[k] = max(worst.get(k, 0.0), res[k])
        print(f"       candidates {lo}..{lo + len(cand) - 1}: {res}", flush=True)
    print(f"       {name}: {n_el} elements, worst over chunks {worst}", flush=True)
