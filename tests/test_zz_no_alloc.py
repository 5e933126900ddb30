"""The entry point that allocates nothing (pskv_attn_bwd_noalloc, for callers that cannot call
hipMalloc: code under graph capture, tight serving loops): called through the C ABI and checked
against pskv_attn_bwd with a workspace of the caller's, bit for bit (both run the same kernels; only
where the B*Hq*S floats between them live differs), and against the CPU oracle - on two calls in a
row, the second on a smaller problem, so that what the first call left in the library's built-in
scratch is still there when the second runs."""
import ctypes

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


def forward_and_dout(pk, inp, seed):
    import torch
    w = inp.w
    d = pu.to_device(inp)
    lse = torch.empty((w.B, w.Hq, w.S), dtype=torch.float32, device="cuda:0")
    out = pk.pskv_attn_fwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], lse=lse, scale=inp.scale)
    dout_host, dout64 = pu.make_dout(inp, seed)
    t = torch.from_numpy(dout_host)
    dout = (t.view(torch.bfloat16) if w.dtype == "bf16" else t).to("cuda:0")
    return d, out, lse, dout, dout64


def raw_noalloc_call(pk, p, d, out, lse, dout, dq, dk, dv):
    """Straight through ctypes: pointers and the params struct, nothing else."""
    import torch
    vp = lambda t: None if t is None else ctypes.c_void_p(t.data_ptr())     # noqa: E731
    rc = pk.load().pskv_attn_bwd_noalloc(ctypes.byref(p), vp(d["q"]), vp(d["k_suf"]), vp(d["v_suf"]), vp(d["k_pre"]),
                                         vp(d["v_pre"]), vp(d["suf_len"]), vp(out), vp(lse), vp(dout), vp(dq), vp(dk),
                                         vp(dv), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    return rc


@pytest.mark.parametrize("shapes", [
    # (B, P, S, lo, hi, Hq, Hkv): first call, then a smaller second call
    [(48, 256, 24, 16, 24, 32, 8), (5, 200, 24, 1, 24, 8, 2)],        # resident dq kernel, the headline shape in small
    [(6, 700, 70, 33, 70, 4, 2), (2, 300, 33, 5, 33, 14, 2)],         # streamed dq kernel, ragged everything
])
def test_noalloc_matches_the_workspace_call_on_two_calls_in_a_row(pk, shapes):
    import torch
    for n, (B, P, S, lo, hi, Hq, Hkv) in enumerate(shapes):
        w = gen.custom_workload(f"noalloc_{B}_{P}_{S}", B, P, S, lo, hi, Hq, Hkv, 128, "bf16", index=1700 + B + P)
        inp = gen.make_inputs(w, pad="nan")
        print(f"[case] no-alloc call {n}: B={B} P={P} S={S} len={lo}..{hi} Hq={Hq} Hkv={Hkv} seed={w.seed}", flush=True)
        d, out, lse, dout, dout64 = forward_and_dout(pk, inp, w.seed + 7)
        nan = float("nan")
        mine = [torch.full_like(d["q"], nan), torch.full_like(d["k_suf"], nan), torch.full_like(d["k_suf"], nan)]
        p = pk.make_params(B, S, P, Hq, Hkv, 128, "bf16", "auto", inp.scale)
        before = torch.cuda.memory_allocated()
        rc = raw_noalloc_call(pk, p, d, out, lse, dout, *mine)
        assert rc == pk.PSKV_OK, pk.pskv_last_error()
        assert torch.cuda.memory_allocated() == before          # nothing taken from torch's allocator either
        torch.cuda.synchronize()
        ws = torch.empty(B * Hq * S * 4, dtype=torch.uint8, device="cuda:0")
        ref = pk.pskv_attn_bwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], out, lse, dout,
                               scale=inp.scale, workspace=ws)
        torch.cuda.synchronize()
        for name, a, b in zip(("dq", "dk_suf", "dv_suf"), mine, ref):
            assert torch.equal(a.view(torch.int16), b.view(torch.int16)), f"{name}: bits differ from pskv_attn_bwd"
        valid = np.arange(S)[None, :] < inp.suf_len[:, None]
        for name, g, r in zip(("dq", "dk_suf", "dv_suf"), mine, pu.oracle_bwd(inp, dout64)):
            pu.compare_grad(pu.out_to_f64(g), r, valid, "bf16", f"no-alloc {name}")


def test_noalloc_through_the_binding_and_its_size_limit(pk):
    import torch
    w = gen.custom_workload("noalloc_bind", 4, 256, 24, 16, 24, 8, 2, 128, "bf16", index=1790)
    inp = gen.make_inputs(w, pad="nan")
    d, out, lse, dout, dout64 = forward_and_dout(pk, inp, 1791)
    grads = [torch.empty_like(d["q"]), torch.empty_like(d["k_suf"]), torch.empty_like(d["k_suf"])]
    pk.pskv_attn_bwd_noalloc(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], out, lse, dout, *grads,
                             scale=inp.scale)
    ref = pk.pskv_attn_bwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], out, lse, dout,
                           scale=inp.scale)
    torch.cuda.synchronize()
    for a, b in zip(grads, ref):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    # beyond the built-in scratch: refused with a clear error before anything is launched (the pointers are
    # never looked at: the tensors of the small problem stand in)
    big = pk.make_params(4096, 64, 512, 40, 40, 128, "bf16", "auto", 0.0)
    rc = raw_noalloc_call(pk, big, d, out, lse, dout, *grads)
    assert rc == pk.PSKV_ERR_WORKSPACE and "exceed" in pk.pskv_last_error()
    # fp32 tensors take the vector-ALU kernels, which use no scratch: served without it
    w32 = gen.custom_workload("noalloc_f32", 3, 21, 9, 0, 9, 4, 2, 64, "f32", index=1792)
    inp32 = gen.make_inputs(w32, pad="nan")
    d32, out32, lse32, dout32, dout64_32 = forward_and_dout(pk, inp32, 1793)
    g32 = [torch.empty_like(d32["q"]), torch.empty_like(d32["k_suf"]), torch.empty_like(d32["k_suf"])]
    pk.pskv_attn_bwd_noalloc(d32["q"], d32["k_suf"], d32["v_suf"], d32["k_pre"], d32["v_pre"], d32["suf_len"], out32, lse32,
                             dout32, *g32, scale=inp32.scale)
    torch.cuda.synchronize()
    valid = np.arange(w32.S)[None, :] < inp32.suf_len[:, None]
    for name, g, r in zip(("dq", "dk_suf", "dv_suf"), g32, pu.oracle_bwd(inp32, dout64_32)):
        pu.compare_grad(pu.out_to_f64(g), r, valid, "f32", f"no-alloc f32 {name}")
