"""GPU parity of guide_simulate against the CPU oracle's step-level simulator."""
import numpy as np
import pytest

from paper_2412_04788_amd import workloads as wl
from tests import bridge

pytestmark = pytest.mark.gpu
TOL = 1e-9
FLOATS = ("ttft_p50", "ttft_p99", "mean_tpot", "tokens_s")


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available()
    return torch


def _run(torch, ctx, grid, cfg_idx, rate, trace, time_model=0, scheduler=0):
    n_cfg = len(cfg_idx)
    out = {k: torch.full((n_cfg,), -1.0, dtype=torch.float64, device="cuda") for k in FLOATS}
    out["status"] = torch.full((n_cfg,), -1, dtype=torch.int32, device="cuda")
    out["n_steps"] = torch.full((n_cfg,), -1, dtype=torch.int64, device="cuda")
    out["n_request_steps"] = torch.full((n_cfg,), -1, dtype=torch.int64, device="cuda")
    ws = torch.empty(ctx.simulate_workspace_bytes(n_cfg, len(trace.n_in)), dtype=torch.uint8, device="cuda")
    d_idx = torch.from_numpy(np.ascontiguousarray(cfg_idx).view(np.int32)).cuda()
    d_rate = torch.from_numpy(np.ascontiguousarray(rate)).cuda()
    ctx.simulate(bridge.gpu_grid(grid), d_idx, d_rate, (trace.arrival_unit, trace.n_in, trace.n_out), out, ws,
                 time_model=time_model, scheduler=scheduler)
    torch.cuda.synchronize()
    res = {k: bridge.to_np(out[k]) for k in FLOATS}
    res["status"] = bridge.to_np(out["status"], np.uint32)
    res["n_steps"] = bridge.to_np(out["n_steps"], np.uint64)
    res["n_request_steps"] = bridge.to_np(out["n_request_steps"], np.uint64)
    return res


def _compare(got, exp):
    np.testing.assert_array_equal(got["status"], exp["status"])
    np.testing.assert_array_equal(got["n_steps"], exp["n_steps"])
    np.testing.assert_array_equal(got["n_request_steps"], exp["n_request_steps"])
    for k in FLOATS:
        e = bridge.rel_err(got[k], exp[k])
        assert e.max() <= TOL, (k, int(e.argmax()), float(e.max()), got[k][e.argmax()], exp[k][e.argmax()])


def test_short_traces_and_ragged_config_counts(ora, torch_cuda):
    torch = torch_cuda
    g = wl.grid_full()
    ctx = bridge.gpu_context(g)
    og = bridge.ora_grid(g)
    for n_req, n_cfg in [(1, 3), (2, 64), (37, 65), (200, 130)]:
        tr = wl.request_trace(n=n_req)
        idx, rate = wl.sim_configs(g, n_cfg, seed=wl.SEED + n_req)
        got = _run(torch, ctx, g, idx, rate, tr)
        exp = ora.simulate_grid(og, idx, rate, tr.arrival_unit, tr.n_in, tr.n_out)
        _compare(got, exp)
        assert (exp["status"] == 0).any()


def test_full_trace_2048_configs(ora, torch_cuda):
    """1024 requests per configuration, configurations drawn from the 1.9M grid."""
    torch = torch_cuda
    g = wl.grid_full()
    ctx = bridge.gpu_context(g)
    tr = wl.request_trace()
    idx, rate = wl.sim_configs(g, 2048)
    got = _run(torch, ctx, g, idx, rate, tr)
    exp = ora.simulate_grid(bridge.ora_grid(g), idx, rate, tr.arrival_unit, tr.n_in, tr.n_out)
    _compare(got, exp)
    ok = exp["status"] == 0
    assert ok.sum() > 1000 and (~ok).sum() > 0
    assert got["n_request_steps"][ok].min() >= tr.n_out.sum()


def test_benchmark_size_sampled_configs_and_invariants(ora, torch_cuda):
    """The benchmark's launch: 65 536 configurations x 1024 requests, both schedulers.  256 configurations spread
    over the list are checked one by one against the oracle; the rest through invariants that hold for any
    schedule (every request emits all its tokens, steps are bounded by tokens, the first 2048 configurations are the
    ones of the 2048-configuration run)."""
    torch = torch_cuda
    g = wl.grid_full()
    ctx = bridge.gpu_context(g)
    og = bridge.ora_grid(g)
    tr = wl.request_trace()
    n_cfg = 65536
    idx, rate = wl.sim_configs(g, n_cfg)
    pick = np.linspace(0, n_cfg - 1, 256).astype(np.int64)
    for sched in (0, 1):
        got = _run(torch, ctx, g, idx, rate, tr, scheduler=sched)
        exp = ora.simulate_grid(og, idx[pick], rate[pick], tr.arrival_unit, tr.n_in, tr.n_out, scheduler=sched)
        _compare({k: v[pick] for k, v in got.items()}, exp)
        ok = got["status"] == 0
        assert ok.sum() > 50000 and set(np.unique(got["status"])) <= {0, 1}
        # decode tokens: every request's n_out - 1 decode steps, plus at least one prompt chunk each
        assert (got["n_request_steps"][ok] >= int((tr.n_out - 1).sum()) + len(tr.n_in)).all()
        assert (got["n_steps"][ok] <= int((tr.n_in + tr.n_out).sum()) + len(tr.n_in)).all()
        assert (got["n_steps"][ok] >= int(tr.n_out.max()) - 1).all()
        assert np.isfinite(got["ttft_p99"][ok]).all() and (got["ttft_p50"][ok] <= got["ttft_p99"][ok]).all()
        assert (got["tokens_s"][ok] > 0).all() and np.isinf(got["ttft_p50"][~ok]).all() and (got["n_steps"][~ok] == 0).all()
        if sched == 0:
            first = _run(torch, ctx, g, idx[:2048], rate[:2048], tr)
            for k in first:
                np.testing.assert_array_equal(first[k], got[k][:2048])


def test_prefill_first_scheduler(ora, torch_cuda):
    """The whole-prompt, decoders-pause variant on the full trace and on a tight pool."""
    torch = torch_cuda
    g = wl.grid_full()
    ctx = bridge.gpu_context(g)
    tr = wl.request_trace()
    idx, rate = wl.sim_configs(g, 1024, seed=wl.SEED + 9)
    got = _run(torch, ctx, g, idx, rate, tr, scheduler=1)
    exp = ora.simulate_grid(bridge.ora_grid(g), idx, rate, tr.arrival_unit, tr.n_in, tr.n_out, scheduler=1)
    _compare(got, exp)
    ok = exp["status"] == 0
    assert ok.sum() > 500
    assert np.all(got["n_request_steps"][ok] == tr.n_out.sum())     # one prompt pass + out - 1 decode tokens each
    split = _run(torch, ctx, g, idx, rate, tr, scheduler=0)
    assert np.any(split["ttft_p99"][ok] != got["ttft_p99"][ok])
    for n_req, n_cfg, tm in [(1, 5, 0), (50, 70, 1)]:
        tr2 = wl.request_trace(n=n_req, seed=3)
        idx2, rate2 = wl.sim_configs(g, n_cfg, seed=77)
        got = _run(torch, ctx, g, idx2, rate2, tr2, time_model=tm, scheduler=1)
        exp = ora.simulate_grid(bridge.ora_grid(g), idx2, rate2, tr2.arrival_unit, tr2.n_in, tr2.n_out, time_model=tm,
                                scheduler=1)
        _compare(got, exp)


def test_tight_pool_odd_values_additive(ora, torch_cuda):
    """Head-of-line blocking on a tight KV pool, odd TP / block / budget values, one-token
    generations, link latency, additive time model."""
    torch = torch_cuda
    m = wl.DENSE_7B
    hws = [wl.Hardware(1e15, 5e12, 2 * 6738149376 + 1200 * 16 * 524288, 4e11, 2e-6),    # pool of 1200 blocks
           wl.Hardware(2e14, 6e12, 40 * wl.GIB, 3e11, 0.0)]
    g = wl.make_grid([m, wl.MOE_8X], hws, wl.Axis.table([1, 3, 50, 1024]), wl.Axis.table([1]), wl.Axis.table([1]),
                     wl.Axis.table([1, 3]), wl.Axis.table([16, 4]), wl.Axis.table([16, 24]),
                     wl.Axis.table([100, 1000, 8192]))
    ctx = bridge.gpu_context(g)
    tr = wl.request_trace(n=300, seed=7)
    n_out = tr.n_out.copy(); n_out[::7] = 1
    tr = wl.Trace(tr.arrival_unit, tr.n_in, n_out)
    idx = np.arange(g.size, dtype=np.uint32)
    rate = np.array([3.0 if i % 2 else 50.0 for i in range(g.size)])
    for tm, sched in ((0, 0), (1, 0), (0, 1)):
        got = _run(torch, ctx, g, idx, rate, tr, time_model=tm, scheduler=sched)
        exp = ora.simulate_grid(bridge.ora_grid(g), idx, rate, tr.arrival_unit, tr.n_in, tr.n_out, time_model=tm,
                                scheduler=sched)
        _compare(got, exp)


def test_bad_index_and_errors(torch_cuda):
    torch = torch_cuda
    from paper_2412_04788_amd import guide
    g = wl.grid_tiny()
    ctx = bridge.gpu_context(g)
    tr = wl.request_trace(n=8)
    idx = np.array([0, g.size, 2 ** 32 - 1], dtype=np.uint32)
    got = _run(torch, ctx, g, idx, np.array([1.0, 1.0, 1.0]), tr)
    assert list(got["status"]) == [0, guide.SIM_BAD_INPUT, guide.SIM_BAD_INPUT]
    bad = wl.Trace(tr.arrival_unit[::-1].copy(), tr.n_in, tr.n_out)
    with pytest.raises(guide.GuideError):
        _run(torch, ctx, g, idx, np.ones(3), bad)
    zero = wl.Trace(tr.arrival_unit, tr.n_in, np.zeros(8, dtype=np.uint32))
    with pytest.raises(guide.GuideError):
        _run(torch, ctx, g, idx, np.ones(3), zero)


def _compare_closed(got, exp):
    """Closed-form runs: times equal to rounding; integer outputs equal unless the oracle saw an admission test
    decided within 1e-9 relative (then the configuration is a listed near-tie, not a failure)."""
    np.testing.assert_array_equal(got["status"], exp["status"])
    same = (got["n_steps"] == exp["n_steps"]) & (got["n_request_steps"] == exp["n_request_steps"])
    near = exp["min_admit_margin"] < TOL
    assert np.all(same | near), np.flatnonzero(~(same | near))[:10]
    for k in FLOATS:
        e = bridge.rel_err(got[k][same], exp[k][same])
        assert e.max() <= TOL, (k, int(e.argmax()), float(e.max()))
    return np.flatnonzero(~same)


@pytest.mark.parametrize("scheduler", [0, 1])
def test_closed_form_runs(ora, torch_cuda, scheduler):
    """GUIDE_SIM_CLOSED_FORM_RUNS against the oracle's closed-form tier, and against the stepped oracle."""
    torch = torch_cuda
    from paper_2412_04788_amd import guide
    g = wl.grid_full()
    ctx = bridge.gpu_context(g)
    og = bridge.ora_grid(g)
    flag = scheduler | guide.SIM_CLOSED_FORM_RUNS
    for n_req, n_cfg, tm in [(1, 3, 0), (2, 64, 0), (37, 65, 1), (200, 130, 0), (1024, 700, 0)]:
        tr = wl.request_trace(n=n_req)
        idx, rate = wl.sim_configs(g, n_cfg, seed=wl.SEED + n_req)
        got = _run(torch, ctx, g, idx, rate, tr, time_model=tm, scheduler=flag)
        exp = ora.simulate_grid(og, idx, rate, tr.arrival_unit, tr.n_in, tr.n_out, time_model=tm,
                                scheduler=scheduler | ora.SIM_CLOSED_FORM_RUNS)
        diverged = _compare_closed(got, exp)
        stepped = ora.simulate_grid(og, idx, rate, tr.arrival_unit, tr.n_in, tr.n_out, time_model=tm, scheduler=scheduler)
        diverged0 = _compare_closed(got, stepped)
        print("closed-form runs", n_req, n_cfg, "near-ties vs closed-form oracle", list(diverged),
              "vs stepped oracle", list(diverged0))
        assert (exp["status"] == 0).any()
    # tight pool, odd values, one-token generations
    m = wl.DENSE_7B
    hws = [wl.Hardware(1e15, 5e12, 2 * 6738149376 + 1200 * 16 * 524288, 4e11, 2e-6),
           wl.Hardware(2e14, 6e12, 40 * wl.GIB, 3e11, 0.0)]
    g2 = wl.make_grid([m, wl.MOE_8X], hws, wl.Axis.table([1, 3, 50, 1024]), wl.Axis.table([1]), wl.Axis.table([1]),
                      wl.Axis.table([1, 3]), wl.Axis.table([16, 4]), wl.Axis.table([16, 24]),
                      wl.Axis.table([100, 1000, 8192]))
    ctx2 = bridge.gpu_context(g2)
    tr = wl.request_trace(n=300, seed=7)
    n_out = tr.n_out.copy(); n_out[::7] = 1
    tr = wl.Trace(tr.arrival_unit, tr.n_in, n_out)
    idx = np.arange(g2.size, dtype=np.uint32)
    rate = np.array([3.0 if i % 2 else 50.0 for i in range(g2.size)])
    got = _run(torch, ctx2, g2, idx, rate, tr, scheduler=flag)
    exp = ora.simulate_grid(bridge.ora_grid(g2), idx, rate, tr.arrival_unit, tr.n_in, tr.n_out,
                            scheduler=scheduler | ora.SIM_CLOSED_FORM_RUNS)
    _compare_closed(got, exp)
