"""The hot calls under HIP graph capture: forward + backward with a plan, and the plan-free forward,
are captured once and replayed several times with eager launches of the same plan in between; every
replay must reproduce the eager result bit for bit.  (The kernels clear their own ticket and arrival
counters when they leave, with stores, not with memset nodes, so a replay always finds them clear.)"""
import numpy as np
import pytest

from paper_2412_01523_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("lens,H", [([700, 1500, 64, 300, 2049], 4), ([6000, 300], 1)],
                         ids=["several-sequences", "cut-tiles"])
def test_forward_backward_replayed_from_a_graph(lens, H):
    import torch
    from paper_2412_01523_amd import binding as fx
    ctx = fx.Context(0)
    D = 128
    cu = wl.cu_seqlens(lens)
    T = int(cu[-1])
    bits = lambda tid: torch.from_numpy(wl.normal_bf16(31337, tid, (T, H, D)).view(np.int16)).view(torch.bfloat16).cuda()
    q, k, v, g = bits(wl.TID_Q), bits(wl.TID_K), bits(wl.TID_V), bits(wl.TID_DO)
    o, dq, dk, dv = (torch.empty_like(q) for _ in range(4))
    lse = torch.empty((H, T), dtype=torch.float32, device="cuda")
    cud = torch.from_numpy(cu).cuda()
    plan = fx.Plan(ctx, cu, H, H, D, True)
    if H == 1:
        items, _ = plan.items(fx.PASS_FWD)
        assert int(items["nparts"].max()) > 1, "the workload was meant to have cut tiles"

    def step(stream):
        fx.flexsp_attn_varlen_fwd(ctx, plan, q, k, v, cud, o, lse, stream=stream)
        fx.flexsp_attn_varlen_bwd(ctx, plan, q, k, v, o, g, lse, cud, dq, dk, dv, stream=stream)

    outs = (o, lse, dq, dk, dv)
    step(torch.cuda.current_stream())   # eager: also completes the plan's upload before the capture
    torch.cuda.synchronize()
    ref = [t.clone() for t in outs]

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        step(torch.cuda.current_stream())
    torch.cuda.synchronize()
    for rep in range(3):
        for t in outs:
            t.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for name, a, b in zip(("O", "LSE", "dQ", "dK", "dV"), ref, outs):
            assert torch.equal(a, b), f"replay {rep}: {name} differs from the eager run"
        step(torch.cuda.current_stream())   # the program's own eager work between replays
        torch.cuda.synchronize()
    plan.close()
    ctx.close()


def test_plan_free_forward_replayed_from_a_graph():
    import torch
    from paper_2412_01523_amd import binding as fx
    ctx = fx.Context(0)
    lens, H, D = [513, 64, 1200, 31], 2, 128
    cu = wl.cu_seqlens(lens)
    T = int(cu[-1])
    bits = lambda tid: torch.from_numpy(wl.normal_bf16(4711, tid, (T, H, D)).view(np.int16)).view(torch.bfloat16).cuda()
    q, k, v = bits(wl.TID_Q), bits(wl.TID_K), bits(wl.TID_V)
    o = torch.empty_like(q)
    lse = torch.empty((H, T), dtype=torch.float32, device="cuda")
    cud = torch.from_numpy(cu).cuda()

    def fwd(stream):
        fx.flexsp_attn_varlen_fwd_static(ctx, q, k, v, cud, o, lse, stream=stream)

    fwd(torch.cuda.current_stream())
    torch.cuda.synchronize()
    ref = (o.clone(), lse.clone())
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        fwd(torch.cuda.current_stream())
    torch.cuda.synchronize()
    for rep in range(3):
        o.zero_()
        lse.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(ref[0], o) and torch.equal(ref[1], lse), f"replay {rep} differs from the eager run"
        fwd(torch.cuda.current_stream())
        torch.cuda.synchronize()
    ctx.close()
