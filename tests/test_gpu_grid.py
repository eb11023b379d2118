"""GPU parity of guide_eval_grid and guide_select against the CPU oracle."""
import numpy as np
import pytest

from paper_2412_04788_amd import workloads as wl
from tests import bridge

pytestmark = pytest.mark.gpu
TOL = 1e-9   # relative, fp64 metrics
FLOAT_COLS = ("t_prefill", "t_decode", "t_batch", "decode_tok_s", "cost")


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available()
    return torch


def _compare(got, exp, where=""):
    for k in FLOAT_COLS:
        e = bridge.rel_err(bridge.to_np(got[k]), exp[k])
        assert e.max() <= TOL, (where, k, int(e.argmax()), float(e.max()))
    np.testing.assert_array_equal(bridge.to_np(got["b_max"], np.uint32), exp["b_max"])
    np.testing.assert_array_equal(bridge.to_np(got["feasible"]), exp["feasible"])


@pytest.mark.parametrize("time_model", [0, 1])
def test_tiny_grid_all_rows(ora, torch_cuda, time_model):
    torch = torch_cuda
    g = wl.grid_tiny()
    ctx = bridge.gpu_context(g)
    out = bridge.metric_buffers(g.size)
    ctx.eval_grid(bridge.gpu_grid(g), 0, g.size, out=out, time_model=time_model)
    torch.cuda.synchronize()
    exp = ora.eval_grid(bridge.ora_grid(g), time_model=time_model)
    _compare(out, exp, "tiny")


def test_tiny_grid_argmin_under_ttft_cap(ora, torch_cuda):
    torch = torch_cuda
    from paper_2412_04788_amd import guide
    g = wl.grid_tiny()
    ctx = bridge.gpu_context(g)
    out = bridge.metric_buffers(g.size)
    ctx.eval_grid(bridge.gpu_grid(g), 0, g.size, out=out)
    idx = torch.empty(3, dtype=torch.int64, device="cuda"); val = torch.empty(3, dtype=torch.float64, device="cuda")
    cnt = torch.empty(1, dtype=torch.int64, device="cuda")
    ws = torch.empty(ctx.select_workspace_bytes(guide.SELECT_TOPK, g.size), dtype=torch.uint8, device="cuda")
    ctx.select(guide.SELECT_TOPK, g.size, out["t_batch"], idx, val, cnt, ws, feasible=out["feasible"],
               constraints=[(out["t_prefill"], wl.TTFT_CAP_S)], k=3)
    torch.cuda.synchronize()
    exp = ora.eval_grid(bridge.ora_grid(g))
    e_idx, e_val, e_cnt = ora.select_topk(exp["t_batch"], exp["feasible"], [(exp["t_prefill"], wl.TTFT_CAP_S)], k=3)
    np.testing.assert_array_equal(bridge.to_np(idx, np.uint64), e_idx[0])
    assert bridge.rel_err(bridge.to_np(val), e_val[0]).max() <= TOL
    assert bridge.to_np(cnt, np.uint64)[0] == e_cnt[0]
    # same selection on the GPU's own columns must be bit-exact
    g_idx, g_val, g_cnt = ora.select_topk(bridge.to_np(out["t_batch"]), bridge.to_np(out["feasible"]),
                                          [(bridge.to_np(out["t_prefill"]), wl.TTFT_CAP_S)], k=3)
    np.testing.assert_array_equal(bridge.to_np(val), g_val[0])
    np.testing.assert_array_equal(bridge.to_np(idx, np.uint64), g_idx[0])


def test_ranges_tails_and_null_columns(ora, torch_cuda):
    torch = torch_cuda
    g = wl.grid_full()
    ctx = bridge.gpu_context(g)
    gg, og = bridge.gpu_grid(g), bridge.ora_grid(g)
    for first, count in [(0, 1), (g.size - 1, 1), (777, 1000), (1234567, 333), (g.size - 4099, 4099)]:
        out = bridge.metric_buffers(count)
        ctx.eval_grid(gg, first, count, out=out)
        torch.cuda.synchronize()
        _compare(out, ora.eval_grid(og, first, count), (first, count))
    # a range large enough for the kernel variant that stores large outputs with the streaming hint, starting and
    # ending inside a tile: its head, its tail and stretches in between, with canaries around the buffers' ends
    first, count = 7, g.size - 20
    out = bridge.metric_buffers(count + 2)
    for v in out.values():
        v.fill_(77)
    view = {k: v[1:count + 1] for k, v in out.items()}
    ctx.eval_grid(gg, first, count, out=view)
    torch.cuda.synchronize()
    for k, v in out.items():
        assert float(v[0]) == 77 and float(v[count + 1]) == 77, k
    for lo, n_rows in [(0, 3000), (count - 3000, 3000), (count // 3, 2000), (1234567, 2000)]:
        part = {k: v[lo:lo + n_rows] for k, v in view.items()}
        _compare(part, ora.eval_grid(og, first + lo, n_rows), (first, count, lo))
    # NULL columns are skipped, others still written
    out = bridge.metric_buffers(500, names=("t_batch", "feasible"))
    ctx.eval_grid(gg, 5000, 500, out=out)
    torch.cuda.synchronize()
    exp = ora.eval_grid(og, 5000, 500)
    assert bridge.rel_err(bridge.to_np(out["t_batch"]), exp["t_batch"]).max() <= TOL
    np.testing.assert_array_equal(bridge.to_np(out["feasible"]), exp["feasible"])
    ctx.eval_grid(gg, 0, 0, out=out)       # count 0: no-op


def test_full_grid_sampled_rows_and_blocks(ora, torch_cuda):
    """1 900 800 configurations in one launch (the benchmarked shape); the oracle
    checks 24 contiguous blocks of 512 rows spread over the grid plus 8192 random rows."""
    torch = torch_cuda
    g = wl.grid_full()
    ctx = bridge.gpu_context(g)
    out = bridge.metric_buffers(g.size)
    ctx.eval_grid(bridge.gpu_grid(g), 0, g.size, out=out)
    torch.cuda.synchronize()
    og = bridge.ora_grid(g)
    host = {k: bridge.to_np(v) for k, v in out.items()}
    host["b_max"] = host["b_max"].view(np.uint32)
    rng = np.random.default_rng(99)
    for first in np.linspace(0, g.size - 512, 24).astype(np.int64):
        exp = ora.eval_grid(og, int(first), 512)
        for k in FLOAT_COLS:
            assert bridge.rel_err(host[k][first:first + 512], exp[k]).max() <= TOL, (k, first)
        np.testing.assert_array_equal(host["b_max"][first:first + 512], exp["b_max"])
        np.testing.assert_array_equal(host["feasible"][first:first + 512], exp["feasible"])
    for idx in rng.integers(0, g.size, 8192):
        exp = ora.eval_grid(og, int(idx), 1)
        for k in FLOAT_COLS:
            assert bridge.rel_err(host[k][idx:idx + 1], exp[k]).max() <= TOL, (k, idx)
        assert host["b_max"][idx] == exp["b_max"][0] and host["feasible"][idx] == exp["feasible"][0]
    # properties that hold at any size
    assert np.all(np.isfinite(host["t_batch"])) and np.all(host["t_batch"] > 0)
    np.testing.assert_allclose(host["t_batch"], host["t_prefill"] + host["t_decode"], rtol=1e-15)
    shape = g.radices
    assert np.all(np.diff(host["t_batch"].reshape(shape), axis=4) > 0)      # longer generation costs more
    fe = host["feasible"].reshape(shape)
    assert np.all(np.diff(fe.astype(np.int8), axis=2) <= 0)                 # larger batch never becomes feasible


def test_efficiency_single_sample(ora, torch_cuda):
    torch = torch_cuda
    g = wl.grid_full()
    ctx = bridge.gpu_context(g)
    out = bridge.metric_buffers(2048)
    ctx.eval_grid(bridge.gpu_grid(g), 900000, 2048, out=out, e_c=[0.83], e_b=[1.07])
    torch.cuda.synchronize()
    _compare(out, ora.eval_grid(bridge.ora_grid(g), 900000, 2048, e_c=0.83, e_b=1.07), "eff")


def test_link_latency_odd_tp_and_long_prompts(ora, torch_cuda):
    """Table axes with values off the powers of two: TP 3 and 6, link latency, prompt
    lengths that leave ragged sub-batches and segments, GQA crossover hardware."""
    torch = torch_cuda
    hws = [wl.Hardware(3.0e14, 6.0e12, 141 * wl.GIB, 4.5e11, 2.5e-6),      # low ridge: attention turns compute bound
           wl.Hardware(9.9e14, 3.35e12, 80 * wl.GIB, 9.0e11, 1.0e-6)]
    g = wl.make_grid(wl.MODELS_FULL, hws, wl.Axis.table([1, 3, 7, 48, 300]), wl.Axis.table([1, 17, 1000, 5000, 20001]),
                     wl.Axis.table([1, 2, 77, 1500]), wl.Axis.table([1, 3, 6, 16]), wl.Axis.table([16, 8, 4]),
                     wl.Axis.table([1, 16, 48]), wl.Axis.table([512, 3000, 8192]))
    ctx = bridge.gpu_context(g)
    out = bridge.metric_buffers(g.size)
    ctx.eval_grid(bridge.gpu_grid(g), 0, g.size, out=out)
    torch.cuda.synchronize()
    _compare(out, ora.eval_grid(bridge.ora_grid(g)), "odd")


def test_argument_errors(torch_cuda):
    from paper_2412_04788_amd import guide
    g = wl.grid_tiny()
    ctx = bridge.gpu_context(g)
    gg = bridge.gpu_grid(g)
    out = bridge.metric_buffers(16)
    with pytest.raises(guide.GuideError) as e:
        ctx.eval_grid(gg, g.size - 3, 4, out=out)
    assert e.value.code == guide.E_RANGE
    with pytest.raises(guide.GuideError) as e:
        ctx.eval_grid(gg, 0, 4, out=None)
    assert e.value.code == guide.E_ARG
    with pytest.raises(guide.GuideError) as e:
        ctx.eval_grid(gg, 0, 4, out=out, time_model=7)
    assert e.value.code == guide.E_ARG
    with pytest.raises(guide.GuideError) as e:
        ctx.eval_grid(gg, 0, 4, out=out, e_c=[0.0], e_b=[1.0])
    assert e.value.code == guide.E_ARG
    bad = wl.make_grid([wl.DENSE_7B], [wl.HW_TINY], wl.Axis.table([1]), wl.Axis.table([0]), wl.Axis.table([1]),
                       wl.Axis.table([1]), wl.Axis.table([16]), wl.Axis.table([16]), wl.Axis.table([2048]))
    with pytest.raises(guide.GuideError):
        ctx.eval_grid(bridge.gpu_grid(bad), 0, 1, out=out)
    fresh = guide.Context(0)
    with pytest.raises(guide.GuideError):
        fresh.eval_grid(gg, 0, 4, out=out)          # no models / hardware registered
    with pytest.raises(guide.GuideError):
        fresh.set_models(np.zeros((1, 8), dtype=np.uint32))
    with pytest.raises(guide.GuideError):
        fresh.set_hardware(np.zeros((1, 5)))


def test_tile_shapes_generic_path_and_table_limits(ora, torch_cuda):
    """Every compiled tile shape, a shape without one (generic kernel), the largest model / hardware
    tables (more coefficient rows than the LDS table holds) and a 64-value axis."""
    torch = torch_cuda
    hws = [wl.Hardware(1e14 * (1 + i), 1e12 * (1 + 0.1 * i), (24 + i) * wl.GIB, 1e11 * (1 + i % 5), 1e-6 * (i % 3))
           for i in range(64)]
    models = list(wl.MODELS_FULL) + [wl.Model("m6", 24, 2048, 16, 4, 8192), wl.Model("m7", 60, 6144, 48, 48, 16384),
                                     wl.Model("m8", 16, 1024, 8, 2, 4096, E=4, k=1)]
    shapes = [(nb, nm) for nb in (1, 2, 3, 4) for nm in (1, 2, 3, 4)] + [(4, 5), (5, 1)]   # the last two: generic kernel
    for nb, nm in shapes:
        blks = [16, 32, 8, 64, 128][:nb]
        mbts = [2048, 512, 8192, 300, 4096][:nm]
        g = wl.make_grid(models, hws[:3], wl.Axis.table([2, 9]), wl.Axis.table([100, 3000]), wl.Axis.table([1, 40]),
                         wl.Axis.table([1, 2, 3, 4, 8]), wl.Axis.table([16, 8, 4]), wl.Axis.table(blks),
                         wl.Axis.table(mbts))
        ctx = bridge.gpu_context(g)
        first, count = 7, g.size - 20
        out = bridge.metric_buffers(count)
        ctx.eval_grid(bridge.gpu_grid(g), first, count, out=out)
        torch.cuda.synchronize()
        _compare(out, ora.eval_grid(bridge.ora_grid(g), first, count), ("shape", nb, nm))
    g = wl.make_grid(models, hws, wl.Axis.table(list(range(1, 65))), wl.Axis.table([640]), wl.Axis.table([33]),
                     wl.Axis.table([2]), wl.Axis.table([16]), wl.Axis.table([16, 32]), wl.Axis.table([2048, 4096, 8192]))
    ctx = bridge.gpu_context(g)
    out = bridge.metric_buffers(g.size)
    ctx.eval_grid(bridge.gpu_grid(g), 0, g.size, out=out)
    torch.cuda.synchronize()
    _compare(out, ora.eval_grid(bridge.ora_grid(g)), "max tables")


def test_cluster_extras(ora, torch_cuda):
    torch = torch_cuda
    hws = [wl.HW_TINY, wl.Hardware(3.0e14, 6.0e12, 48 * wl.GIB, 4.5e11, 2.5e-6)]
    g = wl.make_grid(wl.MODELS_FULL, hws, wl.Axis.table([1, 7, 64]), wl.Axis.table([100, 4000]),
                     wl.Axis.table([1, 2, 500]), wl.Axis.table([1, 2, 3, 8, 16]), wl.Axis.table([16, 4]),
                     wl.Axis.table([16, 48]), wl.Axis.table([2048]))
    ctx = bridge.gpu_context(g)
    for n_gpus, tm in ((8, 0), (3, 1)):
        first, count = 5, g.size - 9
        out = dict(s_max=torch.empty(count, dtype=torch.int32, device="cuda"),
                   dp_max=torch.empty(count, dtype=torch.int32, device="cuda"),
                   max_parallelism=torch.empty(count, dtype=torch.int64, device="cuda"),
                   cluster_tok_s=torch.empty(count, dtype=torch.float64, device="cuda"),
                   paper_tok_s=torch.empty(count, dtype=torch.float64, device="cuda"))
        out.update({k: torch.empty(count, dtype=torch.int32, device="cuda")
                    for k in ("b_adj", "n_sub_batches", "n_segments", "s_adj")})
        ctx.eval_extras(bridge.gpu_grid(g), first, count, n_gpus, out, time_model=tm)
        torch.cuda.synchronize()
        exp = ora.eval_extras_grid(bridge.ora_grid(g), n_gpus, first, count, time_model=tm)
        np.testing.assert_array_equal(bridge.to_np(out["s_max"], np.uint32), exp["s_max"])
        np.testing.assert_array_equal(bridge.to_np(out["dp_max"], np.uint32), exp["dp_max"])
        np.testing.assert_array_equal(bridge.to_np(out["max_parallelism"], np.uint64), exp["max_parallelism"])
        for k in ("b_adj", "n_sub_batches", "n_segments", "s_adj"):
            np.testing.assert_array_equal(bridge.to_np(out[k], np.uint32), exp[k], err_msg=k)
        assert exp["n_segments"].max() > 1 and exp["n_sub_batches"].max() > 1 and (exp["b_adj"] < 64).any()
        for k in ("cluster_tok_s", "paper_tok_s"):
            assert bridge.rel_err(bridge.to_np(out[k]), exp[k]).max() <= TOL, k
    # KV-cache reduction: a kept fraction of every request's entries (0 stands for 1); other values are refused
    from paper_2412_04788_amd import guide
    count = g.size
    kept = dict(b_max_kept=torch.empty(count, dtype=torch.int32, device="cuda"),
                s_max_kept=torch.empty(count, dtype=torch.int32, device="cuda"),
                feasible_kept=torch.empty(count, dtype=torch.uint8, device="cuda"))
    grew = 0
    for keep in (0.0, 1.0, 0.5, 0.2, 1.0 / 3.0, 1e-3):
        ctx.eval_extras(bridge.gpu_grid(g), 0, count, 8, kept, kv_keep=keep)
        torch.cuda.synchronize()
        exp = ora.eval_extras_grid(bridge.ora_grid(g), 8, 0, count, kv_keep=keep if keep else 1.0)
        np.testing.assert_array_equal(bridge.to_np(kept["b_max_kept"], np.uint32), exp["b_max_kept"], err_msg=str(keep))
        np.testing.assert_array_equal(bridge.to_np(kept["s_max_kept"], np.uint32), exp["s_max_kept"], err_msg=str(keep))
        np.testing.assert_array_equal(bridge.to_np(kept["feasible_kept"]), exp["feasible_kept"].astype(np.uint8),
                                      err_msg=str(keep))
        grew += int((exp["feasible_kept"] != 0).sum())
    assert grew > 0
    for bad in (-0.1, 1.5, float("nan")):
        with pytest.raises(guide.GuideError) as err:
            ctx.eval_extras(bridge.gpu_grid(g), 0, count, 8, kept, kv_keep=bad)
        assert err.value.code == guide.E_ARG
    # NULL columns are skipped
    only = dict(dp_max=torch.empty(16, dtype=torch.int32, device="cuda"))
    ctx.eval_extras(bridge.gpu_grid(g), 0, 16, 8, only)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(bridge.to_np(only["dp_max"], np.uint32),
                                  ora.eval_extras_grid(bridge.ora_grid(g), 8, 0, 16)["dp_max"])
