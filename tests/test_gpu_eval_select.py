"""GPU parity of evaluate-and-select in one call (guide_eval_select): the columns against the oracle's
evaluation, the selections against the oracle's selection on the same (GPU-computed) columns, bit for bit."""
import numpy as np
import pytest

from paper_2412_04788_amd import workloads as wl
from tests import bridge

pytestmark = pytest.mark.gpu
TOL = 1e-9
F64_COLS = ("t_prefill", "t_decode", "t_batch", "decode_tok_s", "cost")


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available()
    return torch


def _run(torch, ctx, gg, first, count, out, topk=None, pareto=None, time_model=0, eff=None):
    """topk = dict(objective, k, use_feasible, constraints); pareto = dict(x, y, use_feasible, constraints, capacity).
    Returns ((idx[k], val[k], count) or None, (front idx, front size) or None)."""
    from paper_2412_04788_amd import guide
    sels, bufs = [], {}
    if topk is not None:
        k = topk["k"]
        bufs["ti"] = torch.full((k,), -7, dtype=torch.int64, device="cuda")
        bufs["tv"] = torch.full((k,), -7.0, dtype=torch.float64, device="cuda")
        bufs["tc"] = torch.full((1,), -7, dtype=torch.int64, device="cuda")
        sels.append(ctx.column_select(guide.SELECT_TOPK, topk["objective"], bufs["ti"], bufs["tv"], bufs["tc"],
                                      use_feasible=topk.get("use_feasible", True),
                                      constraints=topk.get("constraints", ()), k=k))
    if pareto is not None:
        cap = pareto.get("capacity", count)
        bufs["pi"] = torch.full((max(cap, 1),), -7, dtype=torch.int64, device="cuda")
        bufs["pc"] = torch.full((1,), -7, dtype=torch.int64, device="cuda")
        sels.append(ctx.column_select(guide.SELECT_PARETO, pareto["x"], bufs["pi"], None, bufs["pc"],
                                      objective_y=pareto["y"], use_feasible=pareto.get("use_feasible", True),
                                      constraints=pareto.get("constraints", ()), capacity=cap))
    if pareto is not None and topk is not None and pareto.get("first", False):
        sels.reverse()
    ws = torch.empty(max(ctx.eval_select_workspace_bytes(sels, count), 1), dtype=torch.uint8, device="cuda")
    kw = {} if eff is None else dict(e_c=eff[0], e_b=eff[1])
    ctx.eval_select(gg, first, count, out, sels, ws, time_model=time_model, **kw)
    torch.cuda.synchronize()
    rt = rp = None
    if topk is not None:
        rt = (bridge.to_np(bufs["ti"], np.uint64), bridge.to_np(bufs["tv"]), int(bridge.to_np(bufs["tc"], np.uint64)[0]))
    if pareto is not None:
        m = int(bridge.to_np(bufs["pc"], np.uint64)[0])
        rp = (bridge.to_np(bufs["pi"], np.uint64)[:min(m, pareto.get("capacity", count))], m)
    return rt, rp


def _check_columns(ora, g, first, count, out, time_model=0, eff=None):
    kw = {} if eff is None else dict(e_c=eff[0], e_b=eff[1])
    exp = ora.eval_grid(bridge.ora_grid(g), first, count, time_model=time_model, **kw)
    host = {}
    for k in F64_COLS:
        if k in out:
            host[k] = bridge.to_np(out[k])
            e = bridge.rel_err(host[k], exp[k])
            assert e.max() <= TOL, (k, first, count, float(e.max()))
    if "b_max" in out:
        np.testing.assert_array_equal(bridge.to_np(out["b_max"], np.uint32), exp["b_max"])
    if "feasible" in out:
        host["feasible"] = bridge.to_np(out["feasible"])
        np.testing.assert_array_equal(host["feasible"], exp["feasible"])
    return host, exp


def _expect_topk(ora, host, topk):
    fe = host["feasible"] if topk.get("use_feasible", True) else None
    cons = [(host[c], cap) for c, cap in topk.get("constraints", ())]
    ei, ev, ec = ora.select_topk(host[topk["objective"]], fe, cons, k=topk["k"])
    return ei[0], ev[0], int(ec[0])


def _expect_pareto(ora, host, pareto):
    fe = host["feasible"].copy() if pareto.get("use_feasible", True) else np.ones(len(host[pareto["x"]]), np.uint8)
    for c, cap in pareto.get("constraints", ()):
        fe &= (host[c] <= cap).astype(np.uint8)
    return ora.pareto_sweep(host[pareto["x"]], host[pareto["y"]], fe)


def _assert_selections(ora, host, topk, pareto, rt, rp):
    if topk is not None:
        ei, ev, ec = _expect_topk(ora, host, topk)
        np.testing.assert_array_equal(rt[0], ei)
        np.testing.assert_array_equal(rt[1], ev)
        assert rt[2] == ec
    if pareto is not None:
        exp = _expect_pareto(ora, host, pareto)
        assert rp[1] == len(exp)
        np.testing.assert_array_equal(rp[0], exp[:pareto.get("capacity", len(exp) + 1)])


def test_tiny_grid_ranges_and_modes(ora, torch_cuda):
    torch = torch_cuda
    g = wl.grid_tiny()
    ctx, gg = bridge.gpu_context(g), bridge.gpu_grid(g)
    topk = dict(objective="cost", k=3, constraints=[("t_prefill", wl.TTFT_CAP_S)])
    pareto = dict(x="t_prefill", y="cost")
    for first, count, tm in [(0, g.size, 0), (1, g.size - 2, 0), (7, 5, 0), (500, 1, 0), (0, g.size, 1), (33, 700, 1)]:
        out = bridge.metric_buffers(count)
        rt, rp = _run(torch, ctx, gg, first, count, out, topk, pareto, time_model=tm)
        host, _ = _check_columns(ora, g, first, count, out, time_model=tm)
        _assert_selections(ora, host, topk, pareto, rt, rp)
    # selections alone, in either order, other columns, k = 1..4 folded and k = 8 through the separate pass
    out = bridge.metric_buffers(g.size)
    for k in (1, 2, 4, 8):
        tk = dict(objective="t_batch", k=k, use_feasible=False, constraints=[("cost", 5.0), ("t_decode", 60.0)])
        rt, _ = _run(torch, ctx, gg, 0, g.size, out, topk=tk)
        host, _ = _check_columns(ora, g, 0, g.size, out)
        _assert_selections(ora, host, tk, None, rt, None)
    pa = dict(x="t_decode", y="decode_tok_s", use_feasible=True, constraints=[("t_prefill", 1.0)], capacity=5, first=True)
    rt, rp = _run(torch, ctx, gg, 0, g.size, out, topk=dict(objective="t_prefill", k=2), pareto=pa)
    host, _ = _check_columns(ora, g, 0, g.size, out)
    _assert_selections(ora, host, dict(objective="t_prefill", k=2), pa, rt, rp)
    # a top-k that reads only the front's two columns is folded into the staircase kernel: objective on either
    # column, constraints on both, with and without the flag column, every partial width
    pa2 = dict(x="t_prefill", y="cost")
    for obj, cons, fe, k in [("cost", [("t_prefill", 0.3), ("cost", 1.0)], True, 4), ("t_prefill", [("cost", 0.05)], False, 1),
                             ("t_prefill", [], True, 2), ("cost", [("cost", -1.0)], True, 3)]:
        tk = dict(objective=obj, k=k, use_feasible=fe, constraints=cons)
        rt, rp = _run(torch, ctx, gg, 0, g.size, out, topk=tk, pareto=pa2)
        host, _ = _check_columns(ora, g, 0, g.size, out)
        _assert_selections(ora, host, tk, pa2, rt, rp)
    # k above 4 beside a front: the pass keeps its own launch (with the row sample riding along) and merges alone;
    # a top-k on a third column beside a front: pass + sample rider, merge beside the finishing kernel
    for tk in (dict(objective="cost", k=8, constraints=[("t_prefill", 0.3)]), dict(objective="t_batch", k=3),
               dict(objective="cost", k=5, use_feasible=False)):
        rt, rp = _run(torch, ctx, gg, 0, g.size, out, topk=tk, pareto=pa2)
        host, _ = _check_columns(ora, g, 0, g.size, out)
        _assert_selections(ora, host, tk, pa2, rt, rp)
    # an efficiency sample
    rt, rp = _run(torch, ctx, gg, 0, g.size, out, topk, pareto, eff=(0.83, 1.21))
    host, _ = _check_columns(ora, g, 0, g.size, out, eff=(0.83, 1.21))
    _assert_selections(ora, host, topk, pareto, rt, rp)
    # nothing passes
    tk0 = dict(objective="cost", k=3, constraints=[("t_prefill", -1.0)])
    rt, rp = _run(torch, ctx, gg, 0, g.size, out, tk0, dict(x="t_prefill", y="cost", constraints=[("cost", -1.0)]))
    assert np.all(rt[0] == ora.NO_INDEX) and np.all(np.isinf(rt[1])) and rt[2] == 0 and rp[1] == 0


def test_full_grid_matches_separate_calls_and_oracle(ora, torch_cuda):
    """The benchmark's step: top-3 by cost under the TTFT cap and the (TTFT, cost) front over 1.9M rows."""
    torch = torch_cuda
    g = wl.grid_full()
    ctx, gg = bridge.gpu_context(g), bridge.gpu_grid(g)
    out = bridge.metric_buffers(g.size)
    topk = dict(objective="cost", k=3, constraints=[("t_prefill", wl.TTFT_CAP_S)])
    pareto = dict(x="t_prefill", y="cost")
    for rep in range(2):                                  # twice on one context: the scratch is reset by each call
        rt, rp = _run(torch, ctx, gg, 0, g.size, out, topk, pareto)
        host = {k: bridge.to_np(v) for k, v in out.items()}
        _assert_selections(ora, host, topk, pareto, rt, rp)
    # columns: sampled rows against the oracle, and all rows against the plain evaluation call
    ref = bridge.metric_buffers(g.size)
    ctx.eval_grid(gg, 0, g.size, out=ref)
    torch.cuda.synchronize()
    for k in out:
        assert torch.equal(out[k], ref[k]), k
    rng = np.random.default_rng(3)
    for first in rng.integers(0, g.size - 64, 40):
        exp = ora.eval_grid(bridge.ora_grid(g), int(first), 64)
        for k in F64_COLS:
            assert bridge.rel_err(host[k][first:first + 64], exp[k]).max() <= TOL, k
    # a ragged range in the middle of tiles
    first, count = 1234567, 400001
    out2 = bridge.metric_buffers(count)
    rt, rp = _run(torch, ctx, gg, first, count, out2, topk, pareto)
    host2 = {k: bridge.to_np(v) for k, v in out2.items()}
    for k in F64_COLS:
        np.testing.assert_array_equal(host2[k], host[k][first:first + count])
    _assert_selections(ora, host2, topk, pareto, rt, rp)


def test_topk_without_stored_columns_and_errors(ora, torch_cuda):
    torch = torch_cuda
    from paper_2412_04788_amd import guide
    g = wl.grid_full()
    ctx, gg = bridge.gpu_context(g), bridge.gpu_grid(g)
    first, count = 0, 300000
    topk = dict(objective="cost", k=3, constraints=[("t_prefill", wl.TTFT_CAP_S)])
    rt, _ = _run(torch, ctx, gg, first, count, {}, topk=topk)          # nothing materialised
    out = bridge.metric_buffers(count)
    ctx.eval_grid(gg, first, count, out=out)
    torch.cuda.synchronize()
    host = {k: bridge.to_np(v) for k, v in out.items()}
    _assert_selections(ora, host, topk, None, rt, None)
    # top-k on a column that is not stored (reduced inside the evaluation, which then also takes the Pareto
    # row sample) together with a Pareto front on stored columns
    part = {k: out[k] for k in ("t_prefill", "cost", "feasible")}
    tk = dict(objective="t_batch", k=4, constraints=[("t_decode", 30.0)])
    pa = dict(x="t_prefill", y="cost")
    for fst, cnt_ in [(first, count), (17, 100003)]:
        sub = {k: v[:cnt_] for k, v in part.items()}
        rt, rp = _run(torch, ctx, gg, fst, cnt_, sub, tk, pa)
        full = bridge.metric_buffers(cnt_)
        ctx.eval_grid(gg, fst, cnt_, out=full)
        torch.cuda.synchronize()
        hostf = {k: bridge.to_np(v) for k, v in full.items()}
        for k in sub:
            assert torch.equal(sub[k], full[k]), k
        _assert_selections(ora, hostf, tk, pa, rt, rp)
    ctx.eval_grid(gg, first, count, out=out)
    torch.cuda.synchronize()
    # the Pareto passes read their columns: missing ones are an argument error
    with pytest.raises(guide.GuideError) as e:
        _run(torch, ctx, gg, first, count, {"cost": out["cost"]}, pareto=dict(x="t_prefill", y="cost"))
    assert e.value.code == guide.E_ARG
    with pytest.raises(guide.GuideError) as e:                         # k = 8 is not folded: needs the columns too
        _run(torch, ctx, gg, first, count, {}, topk=dict(objective="cost", k=8))
    assert e.value.code == guide.E_ARG
    # a grid without a tile kernel for its two fastest axes takes the separate passes
    g5 = wl.make_grid(wl.MODELS_FULL[:1], list(g.hws)[:2], wl.Axis.table([1, 8]), wl.Axis.table([128, 2048]),
                      wl.Axis.table([16, 256]), wl.Axis.table([1, 2]), wl.Axis.table([16]),
                      wl.Axis.table([1, 8, 16, 32, 64]), wl.Axis.table([512, 1024, 2048, 4096, 8192]))
    ctx5, gg5 = bridge.gpu_context(g5), bridge.gpu_grid(g5)
    out5 = bridge.metric_buffers(g5.size)
    pareto = dict(x="t_prefill", y="cost")
    rt, rp = _run(torch, ctx5, gg5, 0, g5.size, out5, topk, pareto)
    host5, _ = _check_columns(ora, g5, 0, g5.size, out5)
    _assert_selections(ora, host5, topk, pareto, rt, rp)
    # zero rows: defined outputs
    rt, rp = _run(torch, ctx, gg, 5, 0, {}, topk, dict(x="t_prefill", y="cost", capacity=4))
    assert np.all(rt[0] == ora.NO_INDEX) and rt[2] == 0 and rp[1] == 0


def test_topk_reduced_inside_the_evaluation_for_other_tile_shapes(ora, torch_cuda):
    """Top-k on columns that are not stored, for several tile shapes, ranges that cut tiles, and both time models."""
    torch = torch_cuda
    hws = [wl.Hardware(1e14 * (1 + i), 1e12 * (1 + 0.3 * i), (40 + 30 * i) * wl.GIB, 1e11 * (1 + i), 1e-6 * i) for i in range(3)]
    for nb, nm in [(1, 1), (3, 2), (4, 4), (2, 2), (1, 4), (4, 1)]:
        g = wl.make_grid(wl.MODELS_FULL[:3], hws, wl.Axis.table([1, 4, 64]), wl.Axis.table([100, 3000, 20000]),
                         wl.Axis.table([1, 40, 500]), wl.Axis.table([1, 2, 8]), wl.Axis.table([16, 4]),
                         wl.Axis.table([16, 32, 8, 64][:nb]), wl.Axis.table([2048, 512, 8192, 300][:nm]))
        ctx, gg = bridge.gpu_context(g), bridge.gpu_grid(g)
        for first, count, tm in [(0, g.size, 0), (5, g.size - 9, 1), (g.size // 2 + 1, 77, 0)]:
            tk = dict(objective="cost", k=4, constraints=[("t_prefill", 0.5), ("t_batch", 100.0)])
            rt, _ = _run(torch, ctx, gg, first, count, {}, topk=tk, time_model=tm)
            out = bridge.metric_buffers(count)
            ctx.eval_grid(gg, first, count, out=out, time_model=tm)
            torch.cuda.synchronize()
            host, _ = _check_columns(ora, g, first, count, out, time_model=tm)
            _assert_selections(ora, host, tk, None, rt, None)
            tk1 = dict(objective="decode_tok_s", k=1, use_feasible=False)        # ties: 0 tokens/s when s_out = 1
            rt, _ = _run(torch, ctx, gg, first, count, {}, topk=tk1, time_model=tm)
            _assert_selections(ora, host, tk1, None, rt, None)


def test_topk_carried_by_the_pareto_passes_ties_and_few_passing_rows(ora, torch_cuda):
    """The top-k that shares the Pareto selection's columns keeps its lists in the staircase kernel: objectives with
    many equal values (TTFT does not depend on the output length or the KV block), caps that leave fewer rows than
    k, caps that exactly equal a stored value, ranges that start inside a tile, both time models, k = 1..4, and
    either column as the objective.  The selections are checked on the columns the GPU stored (their parity with
    the oracle's is the business of the other tests)."""
    torch = torch_cuda
    g = wl.grid_full()
    ctx, gg = bridge.gpu_context(g), bridge.gpu_grid(g)
    n = g.size
    cases = [(0, n, 0), (1536 * 7 + 5, 400_003, 0), (n - 77, 77, 1), (123_456, 20_000, 1)]
    for first, count, tm in cases:
        out = bridge.metric_buffers(count)
        ctx.eval_grid(gg, first, count, out=out, time_model=tm)
        torch.cuda.synchronize()
        host = {k: bridge.to_np(out[k]) for k in F64_COLS}
        host["feasible"] = bridge.to_np(out["feasible"])
        cost, ttft = host["cost"], host["t_prefill"]
        ok = host["feasible"] != 0
        cap_tight = float(np.sort(cost[ok])[2]) if ok.sum() > 2 else 1.0      # exactly three feasible rows at or below
        cap_exact = float(np.median(ttft))                                     # equals a stored value: "<=" must include it
        specs = [dict(objective="t_prefill", k=4, constraints=[("cost", float(np.median(cost)))]),
                 dict(objective="t_prefill", k=3, use_feasible=False),
                 dict(objective="cost", k=4, constraints=[("cost", cap_tight)]),
                 dict(objective="cost", k=2, constraints=[("t_prefill", cap_exact)]),
                 dict(objective="cost", k=1, constraints=[("t_prefill", float(ttft.min()) * 0.5)]),       # nothing passes
                 dict(objective="t_prefill", k=4, constraints=[("t_prefill", float(ttft.min()))])]         # the ties at the least TTFT
        for tk in specs:
            pf = dict(x="t_prefill", y="cost", use_feasible=tk.get("use_feasible", True), capacity=4096)
            rt, rp = _run(torch, ctx, gg, first, count, out, topk=tk, pareto=pf, time_model=tm)
            _assert_selections(ora, host, tk, pf, rt, rp)


def test_profile_aid_times_the_evaluation_kernel(torch_cuda):
    torch = torch_cuda
    g = wl.grid_full()
    ctx, gg = bridge.gpu_context(g), bridge.gpu_grid(g)
    out = bridge.metric_buffers(g.size)
    ctx.profile_enable(3)
    for _ in range(5):                                    # two more than the capacity: not timed, no error
        ctx.eval_grid(gg, 0, g.size, out=out)
    ms = ctx.profile_read(3)
    assert len(ms) == 3 and np.all(ms > 0.005) and np.all(ms < 5.0)
    assert len(ctx.profile_read(3)) == 0
    ctx.profile_enable(4, every=3)                        # launches 0, 3, 6 of 7 are timed
    for _ in range(7):
        ctx.eval_grid(gg, 0, g.size, out=out)
    assert len(ctx.profile_read(4)) == 3
    # a step with a top-k and a Pareto selection over stored columns: all three of its kernels are timed
    ctx.profile_enable(8)
    tk = dict(objective="cost", k=3, constraints=[("t_prefill", 0.2)])
    pf = dict(x="t_prefill", y="cost", capacity=256)
    ref = None
    for _ in range(3):                                    # the third finds two pairs: its evaluation kernel alone is timed
        rt, rp = _run(torch, ctx, gg, 0, g.size, out, topk=tk, pareto=pf)
        ref = ref or (rt, rp)
        np.testing.assert_array_equal(rt[0], ref[0][0])
        np.testing.assert_array_equal(rp[0], ref[1][0])
    ms = ctx.profile_read(8)
    assert len(ms) == 7 and np.all(ms > 0.003) and np.all(ms < 5.0)
    ctx.profile_enable(0)
    rt, rp = _run(torch, ctx, gg, 0, g.size, out, topk=tk, pareto=pf)       # untimed: the same selections
    np.testing.assert_array_equal(rt[0], ref[0][0])
    np.testing.assert_array_equal(rp[0], ref[1][0])
    ctx.eval_grid(gg, 0, g.size, out=out)
    torch.cuda.synchronize()
