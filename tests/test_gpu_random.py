"""Seeded random cases for the selection kernels and for evaluate-and-select: sizes around block and wave
boundaries, heavy ties, NaN / inf, every mix of flag, constraints, k, tile shape, range and stored columns.
Expected values come from the oracle on the same (GPU-computed, where evaluated) columns; everything is exact."""
import numpy as np
import pytest

from paper_2412_04788_amd import workloads as wl
from tests import bridge

pytestmark = pytest.mark.gpu
COLS = ("t_prefill", "t_decode", "t_batch", "decode_tok_s", "cost")


def test_random_selections(ora):
    import torch
    from paper_2412_04788_amd import guide
    ctx = bridge.gpu_context(wl.grid_tiny())
    rng = np.random.default_rng(12345)
    for trial in range(60):
        n = int(rng.choice([1, 2, 63, 64, 65, 255, 256, 257, 1000, 2047, 2048, 2049, 5000, 20000, 100000]))
        mode = rng.integers(0, 3)
        if mode == 0:
            x = rng.integers(-5, 5, n).astype(np.float64); y = rng.integers(-5, 5, n).astype(np.float64)
        elif mode == 1:
            x = rng.random(n); y = 1.0 / (x + 0.01) + rng.random(n) * 0.1
        else:
            x = np.round(rng.lognormal(0, 2, n), 2); y = np.round(rng.lognormal(0, 2, n), 1)
        if rng.random() < 0.3:
            x[rng.integers(0, n, max(1, n // 40))] = np.nan
        if rng.random() < 0.3:
            y[rng.integers(0, n, max(1, n // 40))] = np.inf
        fe = (rng.random(n) < rng.choice([0.0, 0.1, 0.7, 1.0])).astype(np.uint8)
        use_fe = rng.random() < 0.7
        c1 = rng.random(n)
        ncon = int(rng.integers(0, 3))
        caps = [0.5, 0.8]
        cols = [c1, y][:ncon]
        k = int(rng.integers(1, 9))
        dx, dy, dfe, dc1 = (torch.from_numpy(a).cuda() for a in (x, y, fe, c1))
        dcols = [dc1, dy][:ncon]
        idx = torch.full((k,), -7, dtype=torch.int64, device="cuda")
        val = torch.full((k,), -7.0, dtype=torch.float64, device="cuda")
        cnt = torch.full((1,), -7, dtype=torch.int64, device="cuda")
        ws = torch.empty(ctx.select_workspace_bytes(guide.SELECT_TOPK, n), dtype=torch.uint8, device="cuda")
        ctx.select(guide.SELECT_TOPK, n, dx, idx, val, cnt, ws, feasible=dfe if use_fe else None,
                   constraints=list(zip(dcols, caps)), k=k)
        torch.cuda.synchronize()
        ei, ev, ec = ora.select_topk(x, fe if use_fe else None, list(zip(cols, caps)), k=k)
        np.testing.assert_array_equal(bridge.to_np(idx, np.uint64), ei[0], err_msg=f"trial {trial}")
        np.testing.assert_array_equal(bridge.to_np(val), ev[0], err_msg=f"trial {trial}")
        assert int(bridge.to_np(cnt, np.uint64)[0]) == int(ec[0]), trial
        pidx = torch.full((n,), -7, dtype=torch.int64, device="cuda")
        pcnt = torch.full((1,), -7, dtype=torch.int64, device="cuda")
        wsp = torch.empty(ctx.select_workspace_bytes(guide.SELECT_PARETO, n), dtype=torch.uint8, device="cuda")
        ctx.select(guide.SELECT_PARETO, n, dx, pidx, None, pcnt, wsp, objective_y=dy, feasible=dfe if use_fe else None,
                   constraints=list(zip(dcols[:1], caps)), capacity=n)
        torch.cuda.synchronize()
        f = fe.copy() if use_fe else np.ones(n, np.uint8)
        for c, cap in zip(cols[:1], caps):
            f &= (c <= cap).astype(np.uint8)
        exp = ora.pareto_sweep(x, y, f) if n > 3000 else ora.pareto_brute(x, y, f)
        m = int(bridge.to_np(pcnt, np.uint64)[0])
        assert m == len(exp), trial
        np.testing.assert_array_equal(bridge.to_np(pidx, np.uint64)[:m], exp, err_msg=f"trial {trial}")


def test_random_evaluate_and_select(ora):
    import torch
    from paper_2412_04788_amd import guide
    rng = np.random.default_rng(777)
    hws = [wl.Hardware(1e14 * (1 + i), 1e12 * (1 + 0.3 * i), (30 + 40 * i) * wl.GIB, 1e11 * (1 + i), 1e-6 * i) for i in range(3)]
    for trial in range(40):
        nb, nm = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        pick = lambda vals, hi: wl.Axis.table([int(v) for v in rng.choice(vals, int(rng.integers(1, hi)), replace=False)])
        g = wl.make_grid(wl.MODELS_FULL[:int(rng.integers(1, 4))], hws[:int(rng.integers(1, 4))],
                         pick([1, 2, 8, 64, 300], 4), pick([64, 500, 3000, 20000], 4), pick([1, 16, 200, 1000], 4),
                         pick([1, 2, 4, 8], 4), pick([16, 8, 4], 3), wl.Axis.table([16, 32, 8, 64, 128][:nb]),
                         wl.Axis.table([2048, 512, 8192, 300, 4096][:nm]))
        ctx, gg = bridge.gpu_context(g), bridge.gpu_grid(g)
        first = int(rng.integers(0, max(1, g.size // 3)))
        count = int(rng.integers(1, g.size - first + 1))
        tm = int(rng.integers(0, 2))
        full = bridge.metric_buffers(count)
        ctx.eval_grid(gg, first, count, out=full, time_model=tm)
        torch.cuda.synchronize()
        host = {k: bridge.to_np(v) for k, v in full.items()}
        cap_of = lambda col: float(np.quantile(host[col], rng.choice([0.1, 0.5, 0.9, 1.0])))
        kk = int(rng.integers(1, 9))
        tk = dict(obj=str(rng.choice(COLS)), fe=bool(rng.random() < 0.7),
                  cons=[(str(c), cap_of(c)) for c in rng.choice(COLS, int(rng.integers(0, 3)), replace=False)])
        pa = dict(x=str(rng.choice(COLS)), y=str(rng.choice(COLS)), fe=bool(rng.random() < 0.7),
                  cons=[(str(c), cap_of(c)) for c in rng.choice(COLS, int(rng.integers(0, 2)), replace=False)])
        if rng.random() < 0.4:                       # a top-k that shares the front's columns
            tk.update(obj=pa["y"], cons=[(pa["x"], cap_of(pa["x"]))][:int(rng.integers(0, 2))], fe=pa["fe"])
            pa["cons"] = []
        which = int(rng.integers(0, 3))               # 0 both, 1 top-k only, 2 front only
        stored = bool(rng.random() < 0.6) or which != 1 or nb > 4 or nm > 4 or kk > 4
        out = bridge.metric_buffers(count) if stored else {}
        ti = torch.full((kk,), -7, dtype=torch.int64, device="cuda")
        tv = torch.full((kk,), -7.0, dtype=torch.float64, device="cuda")
        tc = torch.full((1,), -7, dtype=torch.int64, device="cuda")
        pi = torch.full((count,), -7, dtype=torch.int64, device="cuda")
        pc = torch.full((1,), -7, dtype=torch.int64, device="cuda")
        sels = []
        if which in (0, 1):
            sels.append(ctx.column_select(guide.SELECT_TOPK, tk["obj"], ti, tv, tc, use_feasible=tk["fe"],
                                          constraints=tk["cons"], k=kk))
        if which in (0, 2):
            sels.append(ctx.column_select(guide.SELECT_PARETO, pa["x"], pi, None, pc, objective_y=pa["y"],
                                          use_feasible=pa["fe"], constraints=pa["cons"], capacity=count))
        if rng.random() < 0.5:
            sels.reverse()
        ws = torch.empty(max(ctx.eval_select_workspace_bytes(sels, count), 1), dtype=torch.uint8, device="cuda")
        ctx.eval_select(gg, first, count, out, sels, ws, time_model=tm)
        torch.cuda.synchronize()
        tag = f"trial {trial} shape {(nb, nm)} range {(first, count)} {tk} {pa} which {which} stored {stored}"
        for k in out:
            assert torch.equal(out[k], full[k]), tag
        if which in (0, 1):
            ei, ev, ec = ora.select_topk(host[tk["obj"]], host["feasible"] if tk["fe"] else None,
                                         [(host[c], cap) for c, cap in tk["cons"]], k=kk)
            np.testing.assert_array_equal(bridge.to_np(ti, np.uint64), ei[0], err_msg=tag)
            np.testing.assert_array_equal(bridge.to_np(tv), ev[0], err_msg=tag)
            assert int(bridge.to_np(tc, np.uint64)[0]) == int(ec[0]), tag
        if which in (0, 2):
            f = host["feasible"].copy() if pa["fe"] else np.ones(count, np.uint8)
            for c, cap in pa["cons"]:
                f &= (host[c] <= cap).astype(np.uint8)
            exp = ora.pareto_sweep(host[pa["x"]], host[pa["y"]], f)
            m = int(bridge.to_np(pc, np.uint64)[0])
            assert m == len(exp), tag
            np.testing.assert_array_equal(bridge.to_np(pi, np.uint64)[:m], exp, err_msg=tag)
