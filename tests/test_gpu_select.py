"""GPU parity of the efficiency sweep, top-k with groups, and the Pareto front."""
import numpy as np
import pytest

from paper_2412_04788_amd import workloads as wl
from tests import bridge

pytestmark = pytest.mark.gpu
TOL = 1e-9
STAT_COLS = ("ttft_mean", "ttft_p10", "ttft_p90", "t_batch_mean", "t_batch_p10", "t_batch_p90", "cost")


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available()
    return torch


def _dev(torch, a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.view(dtype)
    return t.cuda()


def _topk(torch, ctx, obj, k=1, feasible=None, constraints=(), group=None, n_groups=1):
    from paper_2412_04788_amd import guide
    n = obj.numel()
    idx = torch.full((n_groups * k,), -7, dtype=torch.int64, device="cuda")
    val = torch.full((n_groups * k,), -7.0, dtype=torch.float64, device="cuda")
    cnt = torch.full((n_groups,), -7, dtype=torch.int64, device="cuda")
    ws = torch.empty(ctx.select_workspace_bytes(guide.SELECT_TOPK, n, n_groups), dtype=torch.uint8, device="cuda")
    ctx.select(guide.SELECT_TOPK, n, obj, idx, val, cnt, ws, feasible=feasible, constraints=constraints, group=group,
               n_groups=n_groups, k=k)
    torch.cuda.synchronize()
    return (bridge.to_np(idx, np.uint64).reshape(n_groups, k), bridge.to_np(val).reshape(n_groups, k),
            bridge.to_np(cnt, np.uint64))


def _pareto(torch, ctx, x, y, feasible=None, constraints=(), capacity=None):
    from paper_2412_04788_amd import guide
    n = x.numel()
    capacity = n if capacity is None else capacity
    idx = torch.full((max(capacity, 1),), -7, dtype=torch.int64, device="cuda")
    cnt = torch.full((1,), -7, dtype=torch.int64, device="cuda")
    ws = torch.empty(ctx.select_workspace_bytes(guide.SELECT_PARETO, n), dtype=torch.uint8, device="cuda")
    ctx.select(guide.SELECT_PARETO, n, x, idx, None, cnt, ws, objective_y=y, feasible=feasible,
               constraints=constraints, capacity=capacity)
    torch.cuda.synchronize()
    m = int(bridge.to_np(cnt, np.uint64)[0])
    return bridge.to_np(idx, np.uint64)[:min(m, capacity)], m


def test_sweep_parity(ora, torch_cuda):
    torch = torch_cuda
    g = wl.grid_full()
    ctx = bridge.gpu_context(g)
    e_c, e_b = wl.efficiency_pairs()
    og, gg = bridge.ora_grid(g), bridge.gpu_grid(g)
    for first, count in [(0, 300), (1111111, 257), (g.size - 130, 130)]:
        st = bridge.metric_buffers(count, names=STAT_COLS + ("b_max", "feasible"))
        ctx.eval_grid(gg, first, count, stats=st, e_c=e_c, e_b=e_b)
        torch.cuda.synchronize()
        exp = ora.eval_sweep_grid(og, e_c, e_b, first, count)
        for k in STAT_COLS:
            e = bridge.rel_err(bridge.to_np(st[k]), exp[k])
            assert e.max() <= TOL, (k, first, float(e.max()))
        np.testing.assert_array_equal(bridge.to_np(st["b_max"], np.uint32), exp["b_max"])
        np.testing.assert_array_equal(bridge.to_np(st["feasible"]), exp["feasible"])
    # other sample counts exercise the nearest-rank positions: n = 2, 10, 33
    for n in (2, 10, 33):
        st = bridge.metric_buffers(64, names=STAT_COLS)
        ctx.eval_grid(gg, 40000, 64, stats=st, e_c=e_c[:n], e_b=e_b[:n])
        torch.cuda.synchronize()
        exp = ora.eval_sweep_grid(og, e_c[:n], e_b[:n], 40000, 64)
        for k in STAT_COLS:
            assert bridge.rel_err(bridge.to_np(st[k]), exp[k]).max() <= TOL, (k, n)


def test_topk_ties_groups_and_sentinels(ora, torch_cuda):
    torch = torch_cuda
    ctx = bridge.gpu_context(wl.grid_tiny())
    rng = np.random.default_rng(21)
    for n in (1, 63, 64, 65, 1000, 300001):
        obj = rng.integers(-20, 20, n).astype(np.float64)          # heavy exact ties, negative values
        obj[rng.integers(0, n, max(1, n // 50))] = np.nan
        obj[rng.integers(0, n, max(1, n // 100))] = -0.0
        fe = (rng.random(n) < 0.6).astype(np.uint8)
        c1, c2 = rng.random(n), rng.random(n)
        grp = rng.integers(0, 12, n).astype(np.uint32)             # ids 10, 11 fall outside n_groups = 10
        d = dict(obj=_dev(torch, obj), fe=_dev(torch, fe), c1=_dev(torch, c1), c2=_dev(torch, c2),
                 grp=_dev(torch, grp.view(np.int32)))
        cons = [(d["c1"], 0.7), (d["c2"], 0.9)]
        ocons = [(c1, 0.7), (c2, 0.9)]
        for k in (1, 3, 8):
            gi, gv, gc = _topk(torch, ctx, d["obj"], k, d["fe"], cons)
            ei, ev, ec = ora.select_topk(obj, fe, ocons, k=k)
            np.testing.assert_array_equal(gi, ei); np.testing.assert_array_equal(gv, ev)
            np.testing.assert_array_equal(gc, ec)
            gi, gv, gc = _topk(torch, ctx, d["obj"], k, d["fe"], cons, d["grp"], 10)
            ei, ev, ec = ora.select_topk(obj, fe, ocons, group=grp, n_groups=10, k=k)
            np.testing.assert_array_equal(gi, ei); np.testing.assert_array_equal(gv, ev)
            np.testing.assert_array_equal(gc, ec)
    # nothing passes
    obj = _dev(torch, np.arange(10.0)); fe = _dev(torch, np.zeros(10, dtype=np.uint8))
    gi, gv, gc = _topk(torch, ctx, obj, 2, fe)
    assert np.all(gi == ora.NO_INDEX) and np.all(np.isinf(gv)) and gc[0] == 0
    # +inf objective is a valid value and sorts last
    obj = _dev(torch, np.array([np.inf, 3.0, np.inf]))
    gi, gv, gc = _topk(torch, ctx, obj, 3)
    assert list(gi[0]) == [1, 0, 2] and gc[0] == 3


def test_pareto_small_with_ties(ora, torch_cuda):
    torch = torch_cuda
    ctx = bridge.gpu_context(wl.grid_tiny())
    rng = np.random.default_rng(8)
    for trial in range(8):
        n = [1, 2, 64, 500, 2000, 2000, 2000, 5000][trial]
        x = rng.integers(0, 30, n).astype(np.float64)
        y = rng.integers(0, 30, n).astype(np.float64)
        if trial == 4:
            x[:] = 5.0
        if trial == 5:
            y = 100.0 - x
        if trial == 6:
            x = rng.random(n) * 1e-3; y = 1.0 / (x + 1e-4) * (1 + 0.01 * rng.random(n)); x[7] = np.nan
        fe = (rng.random(n) < 0.8).astype(np.uint8)
        got, m = _pareto(torch, ctx, _dev(torch, x), _dev(torch, y), _dev(torch, fe))
        exp = ora.pareto_brute(x, y, fe)
        assert m == len(exp)
        np.testing.assert_array_equal(got, exp)
    # constraint column and capacity smaller than the front
    n = 3000
    x = rng.random(n); y = 1.0 - x; c = rng.random(n)
    got, m = _pareto(torch, ctx, _dev(torch, x), _dev(torch, y), None, [(_dev(torch, c), 0.5)], capacity=10)
    exp = ora.pareto_brute(x, y, (c <= 0.5).astype(np.uint8))
    assert m == len(exp) > 10
    np.testing.assert_array_equal(got, exp[:10])
    # no row passes
    got, m = _pareto(torch, ctx, _dev(torch, x), _dev(torch, y), _dev(torch, np.zeros(n, dtype=np.uint8)))
    assert m == 0 and len(got) == 0


def test_full_grid_select_and_pareto_on_gpu_columns(ora, torch_cuda):
    """Selection over the 1.9M-row grid: the GPU's choice must equal the oracle's
    choice on the same (GPU-computed) columns bit for bit, and the oracle's choice on
    oracle-computed columns except at near-ties (none expected here)."""
    torch = torch_cuda
    g = wl.grid_full()
    ctx = bridge.gpu_context(g)
    out = bridge.metric_buffers(g.size)
    ctx.eval_grid(bridge.gpu_grid(g), 0, g.size, out=out)
    torch.cuda.synchronize()
    host = {k: bridge.to_np(v) for k, v in out.items()}
    for cap in wl.SLO_CAPS_S:
        gi, gv, gc = _topk(torch, ctx, out["cost"], 3, out["feasible"], [(out["t_prefill"], cap)])
        ei, ev, ec = ora.select_topk(host["cost"], host["feasible"], [(host["t_prefill"], cap)], k=3)
        np.testing.assert_array_equal(gi, ei); np.testing.assert_array_equal(gv, ev)
        np.testing.assert_array_equal(gc, ec)
    # per-model winners through the group path
    grp = (np.arange(g.size) // (g.size // len(g.models))).astype(np.int32)
    gi, gv, gc = _topk(torch, ctx, out["t_batch"], 2, out["feasible"], [(out["t_prefill"], 0.2)], _dev(torch, grp), 5)
    ei, ev, ec = ora.select_topk(host["t_batch"], host["feasible"], [(host["t_prefill"], 0.2)],
                                 group=grp.view(np.uint32), n_groups=5, k=2)
    np.testing.assert_array_equal(gi, ei); np.testing.assert_array_equal(gv, ev); np.testing.assert_array_equal(gc, ec)
    got, m = _pareto(torch, ctx, out["t_prefill"], out["cost"], out["feasible"])
    exp = ora.pareto_sweep(host["t_prefill"], host["cost"], host["feasible"])
    assert m == len(exp) > 0
    np.testing.assert_array_equal(got, exp)


def test_full_grid_sweep_then_front_and_slo_argmins(ora, torch_cuda):
    """The uncertainty pipeline at full size: 64-sample sweep over the 1.9M-row grid, the (p90 TTFT, cost) front and
    the cheapest configuration under each p90-TTFT cap.  Selections: GPU against the oracle on the same (GPU-computed)
    columns, bit for bit; columns: blocks of rows against the oracle's sweep."""
    torch = torch_cuda
    g = wl.grid_full()
    ctx = bridge.gpu_context(g)
    e_c, e_b = wl.efficiency_pairs()
    st = bridge.metric_buffers(g.size, names=STAT_COLS + ("b_max", "feasible"))
    ctx.eval_grid(bridge.gpu_grid(g), 0, g.size, stats=st, e_c=e_c, e_b=e_b)
    torch.cuda.synchronize()
    host = {k: bridge.to_np(v) for k, v in st.items()}
    og = bridge.ora_grid(g)
    for first in (0, 777_777, g.size - 96):
        exp = ora.eval_sweep_grid(og, e_c, e_b, first, 96)
        for k in STAT_COLS:
            assert bridge.rel_err(host[k][first:first + 96], exp[k]).max() <= TOL, (k, first)
        np.testing.assert_array_equal(host["feasible"][first:first + 96], exp["feasible"])
    got, m = _pareto(torch, ctx, st["ttft_p90"], st["cost"], st["feasible"])
    exp = ora.pareto_sweep(host["ttft_p90"], host["cost"], host["feasible"])
    assert m == len(exp) > 0
    np.testing.assert_array_equal(got, exp)
    for cap in wl.SLO_CAPS_S:
        gi, gv, gc = _topk(torch, ctx, st["cost"], 1, st["feasible"], [(st["ttft_p90"], cap)])
        ei, ev, ec = ora.select_topk(host["cost"], host["feasible"], [(host["ttft_p90"], cap)], k=1)
        np.testing.assert_array_equal(gi, ei); np.testing.assert_array_equal(gv, ev)
        np.testing.assert_array_equal(gc, ec)


def test_select_on_zero_rows(torch_cuda):
    torch = torch_cuda
    ctx = bridge.gpu_context(wl.grid_tiny())
    empty = torch.empty(0, dtype=torch.float64, device="cuda")
    gi, gv, gc = _topk(torch, ctx, empty, 3)
    assert np.all(gi == 2 ** 64 - 1) and np.all(np.isinf(gv)) and gc[0] == 0
    got, m = _pareto(torch, ctx, empty, empty, capacity=4)
    assert m == 0 and len(got) == 0


def test_pareto_large_front_and_repeated_calls(ora, torch_cuda):
    """A front larger than what the finishing block stages in LDS (global-table path), rows outside the
    sampled range, and several calls in a row on one context (the scratch tables return to neutral)."""
    torch = torch_cuda
    ctx = bridge.gpu_context(wl.grid_tiny())
    rng = np.random.default_rng(17)
    n = 40000
    x = rng.random(n) * 100.0
    x[::997] *= 1e6                                      # far outside the bulk: clamped into the last bin
    x[5::991] *= 1e-9
    y = 1.0e9 - 7.0 * x                                  # strictly decreasing in x: every passing row is on the front
    for rep in range(3):
        fe = (rng.random(n) < 0.9).astype(np.uint8)
        got, m = _pareto(torch, ctx, _dev(torch, x), _dev(torch, y), _dev(torch, fe))
        exp = ora.pareto_sweep(x, y, fe)
        assert m == len(exp) > 4096
        np.testing.assert_array_equal(got, exp)
        xs = rng.integers(0, 50, 3000).astype(np.float64); ys = rng.integers(0, 50, 3000).astype(np.float64)
        got, m = _pareto(torch, ctx, _dev(torch, xs), _dev(torch, ys))
        np.testing.assert_array_equal(got, ora.pareto_brute(xs, ys))


def _sample_rows(n):
    """The rows that the Pareto kernels sample out of n (16 384 strides, one row at a scrambled place in each)."""
    ns = 16384
    stride = n // ns if n > ns else 1
    k = np.arange(min(ns, n), dtype=np.uint64)
    jitter = (((k * np.uint64(2654435761)) & np.uint64(0xFFFFFFFF)) >> np.uint64(8)) % np.uint64(stride)
    return (k * np.uint64(stride) + jitter).astype(np.int64)


def test_pareto_large_front_ties_and_one_crowded_bin(ora, torch_cuda):
    """Large fronts that the finishing blocks share out by bin: (a) rows in identical triples, all on the front
    (order among equal points is by row); (b) a staircase of about 20000 rows that lies beyond the sampled range,
    so that one bin, and with it one block, holds more survivors than fit its LDS staging; (c) a flag column that
    fails every sample row."""
    torch = torch_cuda
    ctx = bridge.gpu_context(wl.grid_tiny())
    n = 30000
    t = (np.arange(n) // 3).astype(np.float64)
    rng = np.random.default_rng(23)
    perm = rng.permutation(n)
    x, y = t[perm], -t[perm]
    got, m = _pareto(torch, ctx, _dev(torch, x), _dev(torch, y))
    exp = ora.pareto_sweep(x, y, None)
    assert m == n == len(exp)
    np.testing.assert_array_equal(got, exp)
    n = 40000
    x = rng.random(n) * 100.0
    y = rng.random(n) * 100.0
    odd = np.setdiff1d(np.arange(n), _sample_rows(n))     # the staircase: the rows that the kernels do not sample
    assert 15000 < len(odd) < 25000
    x[odd] = 1000.0 + odd
    y[odd] = -1.0 * odd
    x[odd[7::7]] = x[odd[6::7][:len(odd[7::7])]]          # some equal x in the staircase: only the lower y stays
    got, m = _pareto(torch, ctx, _dev(torch, x), _dev(torch, y))
    exp = ora.pareto_sweep(x, y, None)
    assert m == len(exp) > 15000
    np.testing.assert_array_equal(got, exp)
    # no sample row passes the filter: nothing is pruned before the finishing blocks, which then drop what a
    # kept row of a lower bin dominates
    n = 300000
    x = np.round(rng.random(n) * 1000.0, 1)
    y = np.round(rng.random(n) * 1000.0, 1)
    fe = np.ones(n, np.uint8)
    fe[_sample_rows(n)] = 0
    got, m = _pareto(torch, ctx, _dev(torch, x), _dev(torch, y), _dev(torch, fe))
    exp = ora.pareto_sweep(x, y, fe)
    assert m == len(exp) > 3
    np.testing.assert_array_equal(got, exp)
    # and a small front straight after, on the same context
    xs = rng.integers(0, 50, 3000).astype(np.float64); ys = rng.integers(0, 50, 3000).astype(np.float64)
    got, m = _pareto(torch, ctx, _dev(torch, xs), _dev(torch, ys))
    np.testing.assert_array_equal(got, ora.pareto_brute(xs, ys))


def test_sweep_other_tile_shapes_and_additive(ora, torch_cuda):
    torch = torch_cuda
    hws = [wl.Hardware(3.0e14, 6.0e12, 141 * wl.GIB, 4.5e11, 2.5e-6)]
    g = wl.make_grid(wl.MODELS_FULL[2:], hws, wl.Axis.table([1, 5, 300]), wl.Axis.table([17, 1000, 20001]),
                     wl.Axis.table([1, 77]), wl.Axis.table([1, 3, 16]), wl.Axis.table([16, 4]),
                     wl.Axis.table([1, 16, 48]), wl.Axis.table([512, 8192]))
    ctx = bridge.gpu_context(g)
    e_c, e_b = wl.efficiency_pairs(n=17)
    for first, count, tm in [(0, g.size, 0), (5, g.size - 11, 1), (100, 1, 0), (7, 6, 0)]:
        st = bridge.metric_buffers(count, names=STAT_COLS + ("b_max", "feasible"))
        ctx.eval_grid(bridge.gpu_grid(g), first, count, stats=st, e_c=e_c, e_b=e_b, time_model=tm)
        torch.cuda.synchronize()
        exp = ora.eval_sweep_grid(bridge.ora_grid(g), e_c, e_b, first, count, time_model=tm)
        for k in STAT_COLS:
            e = bridge.rel_err(bridge.to_np(st[k]), exp[k])
            assert e.max() <= TOL, (k, first, float(e.max()))
        np.testing.assert_array_equal(bridge.to_np(st["b_max"], np.uint32), exp["b_max"])
        np.testing.assert_array_equal(bridge.to_np(st["feasible"]), exp["feasible"])
