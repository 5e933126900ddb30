"""The forward calls, and the backward call with a caller-owned workspace, under HIP graph capture.

The library allocates nothing, keeps no state and reads the suffix lengths on the device, so a
call can be recorded into a graph and replayed; this is how a serving loop would issue the many
small attention launches of one decoding step.  Every replay is checked against the eager result
and, once, against the CPU oracle, with eager work and synchronisations between the replays.
"""
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


@pytest.mark.parametrize("B,P,S,lo,hi,Hq,Hkv", [
    (6, 256, 24, 16, 24, 8, 2),     # resident prefix, pipelined kernel
    (3, 700, 32, 20, 32, 8, 2),     # streamed prefix
    (2, 130, 160, 100, 160, 8, 2),  # passes cut out of one candidate
])
def test_forward_replays_from_a_captured_graph(pk, B, P, S, lo, hi, Hq, Hkv):
    import torch
    w = gen.custom_workload(f"graph_{B}_{P}_{S}", B, P, S, lo, hi, Hq, Hkv, 128, "bf16", index=800 + P)
    inp = gen.make_inputs(w, pad="nan")
    d = pu.to_device(inp)
    print(f"[case] graph capture B={B} P={P} S={S} Hq={Hq} Hkv={Hkv} seed={w.seed}", flush=True)
    args = (d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"])
    eager = pk.pskv_attn_fwd(*args, scale=inp.scale)   # also the first call: one-time set-up happens here
    torch.cuda.synchronize()
    pu.compare(pu.out_to_f64(eager), pu.oracle_out(inp), inp.suf_len, "bf16", w.name)

    out = torch.full_like(eager, float("nan"))
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        pk.pskv_attn_fwd(*args, out=out, scale=inp.scale)
    for rep in range(3):
        out.fill_(float("nan"))
        other = pk.pskv_attn_fwd(*args, scale=inp.scale)   # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), eager.view(torch.int16)), f"replay {rep}"
        assert torch.equal(other.view(torch.int16), eager.view(torch.int16))


def test_new_lengths_are_seen_by_a_replay(pk):
    """suf_len is read on the device at run time: a replay after the lengths changed in place
    computes the new problem."""
    import torch
    w = gen.custom_workload("graph_len", 5, 256, 24, 24, 24, 8, 2, 128, "bf16", index=810)
    inp = gen.make_inputs(w, pad="nan")
    d = pu.to_device(inp)
    args = (d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"])
    pk.pskv_attn_fwd(*args, scale=inp.scale)
    torch.cuda.synchronize()
    out = torch.full_like(d["q"], float("nan"))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=torch.cuda.Stream()):
        pk.pskv_attn_fwd(*args, out=out, scale=inp.scale)
    new_len = np.array([24, 7, 0, 16, 1], dtype=np.int32)
    d["suf_len"].copy_(torch.from_numpy(new_len).to("cuda:0"))
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    inp.suf_len[:] = new_len
    res = pu.compare(pu.out_to_f64(out), pu.oracle_out(inp), inp.suf_len, "bf16", "replay with new lengths")
    print(f"       {res}", flush=True)


def test_backward_replays_from_a_captured_graph(pk):
    """The backward call with a caller-owned workspace allocates nothing either: captured once,
    replayed with eager work between the replays, every replay bit-equal to the eager result."""
    import torch
    w = gen.custom_workload("graph_bwd", 6, 256, 24, 16, 24, 8, 2, 128, "bf16", index=820)
    inp = gen.make_inputs(w, pad="nan")
    d = pu.to_device(inp)
    print(f"[case] graph capture of the backward call B={w.B} P={w.P} S={w.S} seed={w.seed}", flush=True)
    lse = torch.empty((w.B, w.Hq, w.S), dtype=torch.float32, device="cuda:0")
    out = pk.pskv_attn_fwd(d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], lse=lse, scale=inp.scale)
    dout_host, _ = pu.make_dout(inp, w.seed + 7)
    dout = torch.from_numpy(dout_host).view(torch.bfloat16).to("cuda:0")
    ws = torch.empty(w.B * w.Hq * w.S * 4, dtype=torch.uint8, device="cuda:0")
    args = (d["q"], d["k_suf"], d["v_suf"], d["k_pre"], d["v_pre"], d["suf_len"], out, lse, dout)
    eager = pk.pskv_attn_bwd(*args, scale=inp.scale, workspace=ws)
    torch.cuda.synchronize()
    g = [torch.full_like(t, float("nan")) for t in eager]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=torch.cuda.Stream()):
        pk.pskv_attn_bwd(*args, dq=g[0], dk_suf=g[1], dv_suf=g[2], scale=inp.scale, workspace=ws)
    for rep in range(3):
        for t in g:
            t.fill_(float("nan"))
        other = pk.pskv_attn_bwd(*args, scale=inp.scale, workspace=ws)   # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b, c in zip(g, eager, other):
            assert torch.equal(a.view(torch.int16), b.view(torch.int16)), f"replay {rep}"
            assert torch.equal(c.view(torch.int16), b.view(torch.int16))
