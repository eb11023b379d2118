"""guide_select_static (the entry point that allocates nothing) against guide_select, through the C ABI:
two calls in a row per mode, the second with a smaller input, so that what the first call left in the
library's static scratch must not leak into the second.  Bit-exact: both run the same kernels."""
import numpy as np
import pytest

from paper_2412_04788_amd import workloads as wl
from tests import bridge

pytestmark = pytest.mark.gpu


def _dev(torch, a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.view(dtype)
    return t.cuda()


def _outs(torch, n_idx, n_cnt):
    return (torch.full((n_idx,), -7, dtype=torch.int64, device="cuda"),
            torch.full((n_idx,), -7.0, dtype=torch.float64, device="cuda"),
            torch.full((n_cnt,), -7, dtype=torch.int64, device="cuda"))


def _columns(torch, rng, n):
    x = rng.integers(0, 5000, n).astype(np.float64) / 7.0
    y = rng.integers(0, 5000, n).astype(np.float64) / 3.0
    x[rng.integers(0, n, max(1, n // 200))] = np.nan
    fe = (rng.random(n) < 0.7).astype(np.uint8)
    c1 = rng.random(n)
    grp = rng.integers(0, 9, n).astype(np.uint32)
    return dict(x=_dev(torch, x), y=_dev(torch, y), fe=_dev(torch, fe), c1=_dev(torch, c1),
                grp=_dev(torch, grp.view(np.int32)), host=dict(x=x, y=y, fe=fe, c1=c1, grp=grp))


def _both(torch, ctx, mode, n, d, k=1, n_groups=1, grouped=False, capacity=0):
    """The same selection through guide_select (caller workspace) and guide_select_static; returns both results."""
    from paper_2412_04788_amd import guide
    res = []
    for static in (False, True):
        n_idx = max(capacity, 1) if mode == guide.SELECT_PARETO else n_groups * k
        idx, val, cnt = _outs(torch, n_idx, n_groups)
        kw = dict(feasible=d["fe"], constraints=[(d["c1"], 0.8)], k=k, n_groups=n_groups,
                  group=d["grp"] if grouped else None)
        if mode == guide.SELECT_PARETO:
            kw.update(objective_y=d["y"], capacity=capacity)
        if static:
            ctx.select_static(mode, n, d["x"], idx, None if mode == guide.SELECT_PARETO else val, cnt, **kw)
        else:
            ws = torch.empty(ctx.select_workspace_bytes(mode, n, n_groups), dtype=torch.uint8, device="cuda")
            ctx.select(mode, n, d["x"], idx, None if mode == guide.SELECT_PARETO else val, cnt, ws, **kw)
        torch.cuda.synchronize()
        res.append((bridge.to_np(idx, np.uint64), bridge.to_np(val), bridge.to_np(cnt, np.uint64)))
    return res


def test_select_static_matches_select(ora):
    import torch
    from paper_2412_04788_amd import guide
    assert torch.cuda.is_available()
    ctx = bridge.gpu_context(wl.grid_tiny())
    rng = np.random.default_rng(77)
    for n in (300001, 4097):                       # the second call is the smaller one
        d = _columns(torch, rng, n)
        h = d["host"]
        # top-k, one group
        a, b = _both(torch, ctx, guide.SELECT_TOPK, n, d, k=3)
        for u, v in zip(a, b):
            np.testing.assert_array_equal(u, v)
        ei, ev, ec = ora.select_topk(h["x"], h["fe"], [(h["c1"], 0.8)], k=3)
        np.testing.assert_array_equal(b[0], ei[0]); np.testing.assert_array_equal(b[1], ev[0])
        assert b[2][0] == ec[0]
        # top-k with groups
        a, b = _both(torch, ctx, guide.SELECT_TOPK, n, d, k=2, n_groups=9, grouped=True)
        for u, v in zip(a, b):
            np.testing.assert_array_equal(u, v)
        ei, ev, ec = ora.select_topk(h["x"], h["fe"], [(h["c1"], 0.8)], group=h["grp"], n_groups=9, k=2)
        np.testing.assert_array_equal(b[0].reshape(9, 2), ei); np.testing.assert_array_equal(b[2], ec)
        # Pareto front
        a, b = _both(torch, ctx, guide.SELECT_PARETO, n, d, capacity=n)
        m = int(a[2][0])
        assert m == int(b[2][0]) and m > 0
        np.testing.assert_array_equal(a[0][:m], b[0][:m])
        ok = (h["fe"] == 1) & (h["c1"] <= 0.8)
        exp = ora.pareto_sweep(h["x"], h["y"], ok.astype(np.uint8))
        np.testing.assert_array_equal(b[0][:m], exp)
    # n = 0 and the size limit
    idx, val, cnt = _outs(torch, 1, 1)
    ctx.select_static(guide.SELECT_PARETO, 0, None, idx, None, cnt, objective_y=None, capacity=1)
    torch.cuda.synchronize()
    assert int(cnt.item()) == 0
    big = guide.STATIC_SELECT_MAX_ROWS + 1
    col = torch.arange(big, dtype=torch.float64, device="cuda")      # x = y = row: only row 0 is not dominated
    with pytest.raises(guide.GuideError) as e:
        ctx.select_static(guide.SELECT_PARETO, big, col, idx, None, cnt, objective_y=col, capacity=1)
    assert e.value.code == guide.E_RANGE and "static scratch" in str(e.value)
    # at the limit the call is accepted, and a top-k of any size is
    n = guide.STATIC_SELECT_MAX_ROWS
    ctx.select_static(guide.SELECT_PARETO, n, col[:n], idx, None, cnt, objective_y=col[:n], capacity=1)
    torch.cuda.synchronize()
    assert int(cnt.item()) == 1 and int(idx.item()) == 0
    idx3, val3, cnt3 = _outs(torch, 1, 1)
    ctx.select_static(guide.SELECT_TOPK, big, col, idx3, val3, cnt3)
    torch.cuda.synchronize()
    assert int(idx3.item()) == 0 and int(cnt3.item()) == big
