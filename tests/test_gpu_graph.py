"""The benchmark step (guide_eval_select) captured into a HIP graph and replayed: with the tables already on the
device the call only launches kernels, so it can be recorded; every replay must reproduce the eager result."""
import numpy as np
import pytest

from paper_2412_04788_amd import workloads as wl
from tests import bridge

pytestmark = pytest.mark.gpu


def test_step_replays_from_a_graph():
    import torch
    from paper_2412_04788_amd import guide
    g = wl.grid_full()
    n = g.size
    ctx, gg = bridge.gpu_context(g), bridge.gpu_grid(g)
    out = bridge.metric_buffers(n)
    ti = torch.empty(3, dtype=torch.int64, device="cuda")
    tv = torch.empty(3, dtype=torch.float64, device="cuda")
    tc = torch.empty(1, dtype=torch.int64, device="cuda")
    pi = torch.empty(1 << 12, dtype=torch.int64, device="cuda")
    pc = torch.empty(1, dtype=torch.int64, device="cuda")
    sels = [ctx.column_select(guide.SELECT_TOPK, "cost", ti, tv, tc, constraints=[("t_prefill", wl.TTFT_CAP_S)], k=3),
            ctx.column_select(guide.SELECT_PARETO, "t_prefill", pi, None, pc, objective_y="cost", capacity=1 << 12)]
    ws = torch.empty(ctx.eval_select_workspace_bytes(sels, n), dtype=torch.uint8, device="cuda")
    results = (out["cost"], out["t_prefill"], out["feasible"], out["b_max"], ti, tv, tc, pc)

    ctx.eval_select(gg, 0, n, out, sels, ws)
    torch.cuda.synchronize()
    front = int(pc.item())
    ref = [t.clone() for t in results] + [pi[:front].clone()]
    assert front > 0

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        ctx.eval_select(gg, 0, n, out, sels, ws)          # the tables now sit on this stream: the next call uploads nothing
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        ctx.eval_select(gg, 0, n, out, sels, ws)
    for rep in range(3):
        for t in results:
            t.fill_(0)                                       # eager work between the replays
        pi.fill_(-1)
        scratch = torch.rand(1 << 20, device="cuda").sum()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = list(results) + [pi[:front]]
        for a, b in zip(got, ref):
            assert torch.equal(a, b), rep
        assert float(scratch) > 0
