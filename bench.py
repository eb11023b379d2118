#!/usr/bin/env python3
"""Benchmark of the GUIDE optimiser hot path on one MI355X.

One step = one pass of the hot path over the full factorial grid (1 900 800
configurations) through one guide_eval_select call: all seven columns are
evaluated and stored, the top-3 by cost under the 200 ms TTFT cap are selected,
and the (TTFT, cost) Pareto front is extracted.  The headline value is
configurations per second over the timed steps, inputs resident in HBM.  The other kernels (efficiency sweep, sampled space, serving simulation)
are timed once each after the steps and reported under "extra".
Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
BYTES_PER_CONFIG = 45           # 5 fp64 + u32 + u8 written per configuration, nothing read
VECTOR_ISSUE_PEAK = 256 * 4 * 16 * 2.4e9      # lane-instructions per second: 256 CU x 4 SIMD x 16 lanes x 2.4 GHz

# Figures taken from rocprofv3 counter runs (profiles/*.md), each with the SHA-256 (first 16 hex digits) of the
# kernel sources it was measured on.  A figure is reported only while those sources are unchanged, else null.
COUNTERS = {
    # in-step launches (with the row-sample blocks): WRITE_SIZE 83594.39 KiB x 1.0 + FETCH_SIZE 259.32 KiB x 2.0 per
    # launch (scales from a 512 MiB device copy): profiles/eval_tile_kernel_full_grid_pmc.md
    "eval_tile_traffic_bytes": {"value": 86_131_743, "sources": ("eval_grid.hip", "perf_model.hpp"),
                                "sha16": "e6fb412dd396ef0b"},
    # SQ_INSTS_VALU 5.138e9 x 64 / 41.08 ms / 39.32e12 for simulate_kernel, split-fuse, stepped:
    # profiles/extra_kernels_valu_pmc.md
    "simulate_vector_issue_frac": {"value": 0.204, "sources": ("simulate.hip", "perf_model.hpp"), "sha16": "78cd9103d96c831d"},
}


def _sources_sha16(names):
    import hashlib
    h = hashlib.sha256()
    for n in names:
        with open(os.path.join(ROOT, "paper_2412_04788_amd", "csrc", n), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def counter_figure(key):
    """The profiled figure, or None once the kernel's sources differ from the ones it was measured on."""
    c = COUNTERS[key]
    return c["value"] if _sources_sha16(c["sources"]) == c["sha16"] else None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-extra", action="store_true", help="skip the sweep / sampled / simulation timings")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--probe", action="store_true",
                    help="counter probe for rocprofv3 --pmc: 10 steps, 10 plain grid evaluations, then 10 plain device copies of "
                         "512 MiB (a kernel of known traffic that calibrates FETCH_SIZE / WRITE_SIZE), no timing")
    ap.add_argument("--probe-extra", action="store_true",
                    help="counter probe: the sweep (1.9M x 64), the sampled space (2^28) and the simulation "
                         "(65 536 configs) only")
    ap.add_argument("--probe-fronts", action="store_true",
                    help="times guide_select PARETO over 1 900 800 synthetic rows whose front has 100 ... 1 900 800 "
                         "members (a dominated cloud plus a staircase), one JSON line")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: the library runs on ONE GPU (no sharding, no collectives); use --gpus 1")

    import numpy as np
    import torch
    from paper_2412_04788_amd import guide, workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    g = wl.grid_full()
    n = g.size
    ctx = guide.Context(0)
    ctx.set_models(wl.models_array(g.models))
    ctx.set_hardware(wl.hw_array(g.hws))
    gg = guide.GridArg([(a.values, a.geom2_start) for a in g.axes])
    dt = {"b_max": torch.int32, "feasible": torch.uint8}
    out = {k: torch.empty(n, dtype=dt.get(k, torch.float64), device="cuda") for k in guide.METRIC_COLUMNS}
    k_top = 3
    sel_idx = torch.empty(k_top, dtype=torch.int64, device="cuda")
    sel_val = torch.empty(k_top, dtype=torch.float64, device="cuda")
    sel_cnt = torch.empty(1, dtype=torch.int64, device="cuda")
    par_cap = 1 << 16
    par_idx = torch.empty(par_cap, dtype=torch.int64, device="cuda")
    par_cnt = torch.empty(1, dtype=torch.int64, device="cuda")
    ws_top = torch.empty(ctx.select_workspace_bytes(guide.SELECT_TOPK, n), dtype=torch.uint8, device="cuda")
    ws_par = torch.empty(ctx.select_workspace_bytes(guide.SELECT_PARETO, n), dtype=torch.uint8, device="cuda")

    # one C call per step, arguments marshalled once
    selections = [
        ctx.column_select(guide.SELECT_TOPK, "cost", sel_idx, sel_val, sel_cnt, use_feasible=True,
                          constraints=[("t_prefill", wl.TTFT_CAP_S)], k=k_top),
        ctx.column_select(guide.SELECT_PARETO, "t_prefill", par_idx, None, par_cnt, objective_y="cost",
                          use_feasible=True, capacity=par_cap),
    ]
    ws_step = torch.empty(ctx.eval_select_workspace_bytes(selections, n), dtype=torch.uint8, device="cuda")
    step = ctx.prepared("eval_select", gg, 0, n, out, selections, ws_step)
    # the same work as three separate calls (timed outside the timed region, for the phase split)
    call_eval = ctx.prepared("eval_grid", gg, 0, n, out=out)
    call_topk = ctx.prepared("select", guide.SELECT_TOPK, n, out["cost"], sel_idx, sel_val, sel_cnt, ws_top,
                             feasible=out["feasible"], constraints=[(out["t_prefill"], wl.TTFT_CAP_S)], k=k_top)
    call_pareto = ctx.prepared("select", guide.SELECT_PARETO, n, out["t_prefill"], par_idx, None, par_cnt, ws_par,
                               objective_y=out["cost"], feasible=out["feasible"], capacity=par_cap)

    if args.probe_fronts:
        print(json.dumps({"probe_fronts": front_timings(ctx, n, torch, np, guide)}))
        return
    if args.probe_extra:
        extra = extra_timings(ctx, gg, g, torch, np, guide, wl)
        print(json.dumps({"probe_extra": extra}))
        return
    if args.probe:
        src = torch.ones(1 << 26, dtype=torch.float64, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(10):
            step()
        for _ in range(10):
            call_eval()
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"probe": "10 x eval_select and 10 x eval_grid over %d configs, 10 x device copy of %d bytes" % (n, src.numel() * 8)}))
        return

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # timed region: exactly K steps, nothing else
    t0 = time.perf_counter()
    for k in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    total = t1 - t0
    # Duration of the grid-evaluation kernel INSIDE the step, in the steady state of the timed region: a second run
    # of the same steps in which the library attaches a pair of HIP events to the dispatch of each of the three
    # kernels of every 8th step, on the launch stream.  A timed launch delays the launches around it by a few
    # microseconds; with seven untimed steps between two timed ones the stream stays as busy as in the
    # throughput run (timing every step leaves the GPU idle before each step, and the evaluation kernel then
    # reads about 1 us shorter -- reported beside it, not used).
    n_timed, every = max(args.steps, 32), 8
    ctx.profile_enable(3 * n_timed, every)
    for k in range(n_timed * every):
        step()
    torch.cuda.synchronize()
    ms_all = np.asarray(ctx.profile_read(3 * n_timed), dtype=np.float64)
    assert ms_all.size == 3 * n_timed
    ms_all = ms_all.reshape(n_timed, 3)             # evaluation (+ row sample), filter (+ top-k lists), finish (+ merge)
    ms_kernel = ms_all[:, 0]
    ms_eval = float(np.mean(ms_kernel))
    ctx.profile_enable(3 * n_timed, 1)
    for k in range(n_timed):
        step()
    torch.cuda.synchronize()
    ms_eval_every_step = float(np.asarray(ctx.profile_read(3 * n_timed), dtype=np.float64).reshape(n_timed, 3)[:, 0].mean())
    ctx.profile_enable(0)
    # the plain evaluation kernel launched back to back between one pair of events (no markers between launches)
    ev2 = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ev2[0].record()
    for _ in range(50):
        call_eval()
    ev2[1].record()
    torch.cuda.synchronize()
    ms_eval_b2b = ev2[0].elapsed_time(ev2[1]) / 50
    # the same step as three separate calls, and the two selections alone
    ev3 = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    reps = 20
    ev3[0].record()
    for _ in range(reps):
        call_eval()
        call_topk()
        call_pareto()
    ev3[1].record()
    for _ in range(reps):
        call_topk()
    ev3[2].record()
    for _ in range(reps):
        call_pareto()
    ev3[3].record()
    torch.cuda.synchronize()
    ms_separate = ev3[0].elapsed_time(ev3[1]) / reps
    ms_topk = ev3[1].elapsed_time(ev3[2]) / reps
    ms_pareto = ev3[2].elapsed_time(ev3[3]) / reps
    step()
    torch.cuda.synchronize()
    value = n * args.steps / total
    achieved = BYTES_PER_CONFIG * n / (ms_eval * 1e-3) / 1e9
    sustained = grid_sustained(torch, guide, wl)

    result = {
        "metric": "configs evaluated/sec (fp64 grid)", "value": value, "unit": "configs/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": total / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": "full factorial grid, 1900800 configs (5 models x 6 hw x 11 batch x 10 s_in x 8 s_out "
                               "x 4 tp x 3 wbits x 2 kv_block x 3 mbt): evaluate all columns + top-3 by cost under 200 ms TTFT + "
                               "(TTFT, cost) Pareto front, one guide_eval_select call",
                   "configs_per_step": n, "top_k": k_top,
                   "selected": [int(v) for v in sel_idx.cpu().numpy().view(np.uint64)],
                   "pareto_front_size": int(par_cnt.item())},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": counter_figure("eval_tile_traffic_bytes"),
                     "kernel": "eval_tile_kernel<false,2,3,false,true>",
                     "kernel_ms": ms_eval, "kernel_ms_min": float(np.min(ms_kernel)),
                     "kernel_launches_timed": n_timed,
                     "timing": "HIP event pairs on the dispatches of the three kernels of every 8th step of a run of 8 x kernel_launches_timed steps",
                     "kernel_ms_when_every_step_is_timed": ms_eval_every_step,
                     "plain_eval_kernel_ms_back_to_back": ms_eval_b2b,
                     "frac_back_to_back": BYTES_PER_CONFIG * n / (ms_eval_b2b * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "bytes_per_config": BYTES_PER_CONFIG, "grid_sustained": sustained},
        "phases_ms": {"eval_kernel_in_step": ms_eval, "filter_topk_kernel_in_step": float(ms_all[:, 1].mean()),
                      "finish_merge_kernel_in_step": float(ms_all[:, 2].mean()),
                      "step_kernels_sum": float(ms_all.sum(axis=1).mean()), "step_as_three_calls": ms_separate,
                      "select_topk_alone": ms_topk, "select_pareto_alone": ms_pareto},
    }

    host = {k: v.cpu().numpy() for k, v in out.items()}
    front = par_idx.cpu().numpy().view(np.uint64)[:min(int(par_cnt.item()), par_cap)]
    result["near_ties"] = near_ties(np, host, sel_idx.cpu().numpy().view(np.uint64), front, wl.TTFT_CAP_S)
    if not args.no_extra:
        result["extra"] = extra_timings(ctx, gg, g, torch, np, guide, wl)
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(g, np, wl, host, result["config"]["selected"], front)
    print(json.dumps(result))


def grid_sustained(torch, guide, wl, n_hw=64, reps=10):
    """The same evaluation kernel on a grid with 64 hardware rows instead of 6 (20 275 200 configurations, 912 MB
    of columns per launch), back to back: the fixed cost of a launch is amortised, what is left is the rate at
    which the kernel computes and stores."""
    g0 = wl.grid_full()
    rng_hw = [wl.Hardware(h.peak_flops * (1.0 + 0.01 * (i // 6)), h.hbm_bw, h.cap_bytes, h.link_bw, h.link_lat)
              for i in range(n_hw) for h in [g0.hws[i % 6]]]
    g = wl.make_grid(g0.models, rng_hw, *g0.axes[2:])
    n = g.size
    ctx = guide.Context(0)
    ctx.set_models(wl.models_array(g.models))
    ctx.set_hardware(wl.hw_array(g.hws))
    gg = guide.GridArg([(a.values, a.geom2_start) for a in g.axes])
    dt = {"b_max": torch.int32, "feasible": torch.uint8}
    out = {k: torch.empty(n, dtype=dt.get(k, torch.float64), device="cuda") for k in guide.METRIC_COLUMNS}
    call = ctx.prepared("eval_grid", gg, 0, n, out=out)
    s = _timed(torch, call, reps=reps)
    del out
    gbs = BYTES_PER_CONFIG * n / s / 1e9
    # what a plain fill of as many bytes reaches on this GPU (a store-only kernel that computes nothing)
    flat = torch.empty(BYTES_PER_CONFIG * n // 8, dtype=torch.float64, device="cuda")
    s_fill = _timed(torch, lambda: flat.fill_(1.0), reps=reps)
    fill_gbs = flat.numel() * 8 / s_fill / 1e9
    return {"configs": n, "kernel_ms": s * 1e3, "configs_per_s": n / s, "achieved_GBs": gbs, "frac": gbs / HBM_PEAK_GBS,
            "plain_fill_same_bytes_GBs": fill_gbs, "frac_of_plain_fill": gbs / fill_gbs}


def near_ties(np, host, top_idx, front, ttft_cap, tol=1e-9):
    """Near-ties of the step's selections on the columns the GPU stored: selected rows whose objective is within
    `tol` (relative) of the next candidate's, passing or failing rows whose TTFT sits within `tol` of the cap,
    and front members with a neighbour within `tol` in either coordinate.  Each is a place where a result may
    differ from a reference evaluation by rounding alone."""
    cost, ttft, fe = host["cost"], host["t_prefill"], host["feasible"] != 0
    ok = fe & (ttft <= ttft_cap)
    cand = np.flatnonzero(ok)
    order = cand[np.lexsort((cand, cost[cand]))][:len(top_idx) + 1]          # k + 1 best by (cost, row)
    vals = cost[order]
    gaps = np.abs(np.diff(vals)) / np.maximum(np.abs(vals[1:]), 1e-300)
    topk = [dict(rows=[int(order[i]), int(order[i + 1])], relative_gap=float(gp)) for i, gp in enumerate(gaps)
            if gp <= tol and cost[order[i]] != cost[order[i + 1]]]
    at_cap = np.flatnonzero(fe & (np.abs(ttft - ttft_cap) <= tol * ttft_cap))
    fx, fy = ttft[front.astype(np.int64)], cost[front.astype(np.int64)]
    if len(front) > 1:
        dx = np.abs(np.diff(fx)) / np.maximum(np.abs(fx[1:]), 1e-300)
        dy = np.abs(np.diff(fy)) / np.maximum(np.abs(fy[1:]), 1e-300)
        close = np.flatnonzero(((dx <= tol) & (dx > 0)) | ((dy <= tol) & (dy > 0)))
    else:
        close = np.zeros(0, dtype=np.int64)
    return {"tolerance": tol, "top_k": topk, "rows_with_ttft_at_cap": [int(i) for i in at_cap[:16]],
            "front_neighbours": [[int(front[i]), int(front[i + 1])] for i in close[:16]],
            "selection_order_matches_columns": bool(np.array_equal(order[:len(top_idx)], top_idx.astype(np.int64)))}


def _timed(torch, fn, reps=1):
    fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps * 1e-3


def front_timings(ctx, n, torch, np, guide, sizes=(100, 1000, 4000, 5000, 20000, 100000, 400000, 1000000, 1900800)):
    """Pareto selection over n rows: `front` of them form a staircase (x up, y down), the others a cloud that the
    staircase dominates.  Fronts of more than 4096 rows take the finishing kernel's many-block path."""
    rng = np.random.default_rng(1)
    res = []
    out_idx = torch.empty(n, dtype=torch.int64, device="cuda")
    cnt = torch.empty(1, dtype=torch.int64, device="cuda")
    ws = torch.empty(ctx.select_workspace_bytes(guide.SELECT_PARETO, n), dtype=torch.uint8, device="cuda")
    for front in sizes:
        front = min(front, n)
        x = rng.random(n) + 2.0
        y = rng.random(n) + 2.0
        idx = rng.choice(n, front, replace=False)
        t = np.sort(rng.random(front))
        x[idx] = t
        y[idx] = 1.0 - t
        dx, dy = torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()
        call = ctx.prepared("select", guide.SELECT_PARETO, n, dx, out_idx, None, cnt, ws, objective_y=dy, capacity=n)
        s = _timed(torch, call, reps=5)
        m = int(cnt.item())
        got = out_idx[:m].cpu().numpy()
        res.append({"front": front, "ms": s * 1e3, "count": m,
                    "rows_match": bool(m == front and np.array_equal(np.sort(got), np.sort(idx)))})
    return res


def extra_timings(ctx, gg, g, torch, np, guide, wl, n_sampled=1 << 28, n_sim=65536):
    """Sweep (1.9M x 64 samples), sampled space (2^28), serving simulation (65 536 x 1024 requests)."""
    n = g.size
    extra = {}
    e_c, e_b = wl.efficiency_pairs()
    dt = {"b_max": torch.int32, "feasible": torch.uint8}
    st = {k: torch.empty(n, dtype=dt.get(k, torch.float64), device="cuda") for k in guide.STATS_COLUMNS}
    s = _timed(torch, lambda: ctx.eval_grid(gg, 0, n, stats=st, e_c=e_c, e_b=e_b))
    extra["sweep"] = {"evaluations_per_s": n * 64 / s, "configs_per_s": n / s, "seconds": s, "samples": 64}
    # the whole uncertainty pipeline: sweep, (p90 TTFT, cost) front, cheapest configuration under each p90-TTFT cap
    p_idx = torch.empty(1 << 16, dtype=torch.int64, device="cuda")
    p_cnt = torch.empty(1, dtype=torch.int64, device="cuda")
    a_idx = torch.empty(len(wl.SLO_CAPS_S), dtype=torch.int64, device="cuda")
    a_val = torch.empty(len(wl.SLO_CAPS_S), dtype=torch.float64, device="cuda")
    a_cnt = torch.empty(len(wl.SLO_CAPS_S), dtype=torch.int64, device="cuda")
    ws_p = torch.empty(ctx.select_workspace_bytes(guide.SELECT_PARETO, n), dtype=torch.uint8, device="cuda")
    ws_t = torch.empty(ctx.select_workspace_bytes(guide.SELECT_TOPK, n), dtype=torch.uint8, device="cuda")

    def pipeline():
        ctx.eval_grid(gg, 0, n, stats=st, e_c=e_c, e_b=e_b)
        ctx.select(guide.SELECT_PARETO, n, st["ttft_p90"], p_idx, None, p_cnt, ws_p, objective_y=st["cost"],
                   feasible=st["feasible"], capacity=1 << 16)
        for j, cap in enumerate(wl.SLO_CAPS_S):
            ctx.select(guide.SELECT_TOPK, n, st["cost"], a_idx[j:j + 1], a_val[j:j + 1], a_cnt[j:j + 1], ws_t,
                       feasible=st["feasible"], constraints=[(st["ttft_p90"], cap)], k=1)
    s = _timed(torch, pipeline, reps=3)
    extra["sweep_pipeline"] = {"configs_per_s": n / s, "seconds": s, "front_size": int(p_cnt.item()),
                               "argmin_under_p90_ttft_caps": [int(v) for v in a_idx.cpu().numpy().view(np.uint64)],
                               "caps_s": list(wl.SLO_CAPS_S)}
    del st

    ex = dict(s_max=torch.empty(n, dtype=torch.int32, device="cuda"),
              dp_max=torch.empty(n, dtype=torch.int32, device="cuda"),
              max_parallelism=torch.empty(n, dtype=torch.int64, device="cuda"),
              cluster_tok_s=torch.empty(n, dtype=torch.float64, device="cuda"),
              paper_tok_s=torch.empty(n, dtype=torch.float64, device="cuda"))
    s = _timed(torch, lambda: ctx.eval_extras(gg, 0, n, 8, ex), reps=5)
    extra["cluster_extras"] = {"configs_per_s": n / s, "seconds": s, "n_gpus": 8, "bytes_per_config": 32}
    del ex

    sp = wl.sample_space()
    space = {f: getattr(sp, f) for f in ("heads", "peak", "bw", "cap", "batch", "s_in", "s_out", "tp", "wbits",
                                         "kv_block", "mbt", "kv_choices", "layers_lo", "layers_n", "ffn_lo_x2",
                                         "ffn_span_x2", "vocab", "link_div")}
    so = dict(feasible_count=torch.empty(1, dtype=torch.int64, device="cuda"),
              win_val=torch.empty(wl.N_BUCKETS, dtype=torch.float64, device="cuda"),
              win_idx=torch.empty(wl.N_BUCKETS, dtype=torch.int64, device="cuda"),
              hist=torch.empty(256, dtype=torch.int64, device="cuda"))
    n_s = n_sampled
    s = _timed(torch, lambda: ctx.eval_sampled(space, wl.SEED, 0, n_s, wl.BUCKET_EDGES, wl.TTFT_CAP_S, so))
    extra["sampled"] = {"configs_per_s": n_s / s, "seconds": s, "candidates": n_s,
                        "feasible": int(so["feasible_count"].item())}

    n_cfg = n_sim
    idx, rate = wl.sim_configs(g, n_cfg)
    tr = wl.request_trace()
    d_idx = torch.from_numpy(idx.view(np.int32)).cuda()
    d_rate = torch.from_numpy(rate).cuda()
    sim = {k: torch.empty(n_cfg, dtype=torch.float64, device="cuda") for k in ("ttft_p50", "ttft_p99", "mean_tpot", "tokens_s")}
    sim["status"] = torch.empty(n_cfg, dtype=torch.int32, device="cuda")
    sim["n_steps"] = torch.empty(n_cfg, dtype=torch.int64, device="cuda")
    sim["n_request_steps"] = torch.empty(n_cfg, dtype=torch.int64, device="cuda")
    ws = torch.empty(ctx.simulate_workspace_bytes(n_cfg, len(tr.n_in)), dtype=torch.uint8, device="cuda")
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    ctx.simulate(gg, d_idx, d_rate, (tr.arrival_unit, tr.n_in, tr.n_out), sim, ws)
    b.record()
    torch.cuda.synchronize()
    s = a.elapsed_time(b) * 1e-3
    rs = int(sim["n_request_steps"].sum().item())
    steps = int(sim["n_steps"].sum().item())
    extra["simulate"] = {"request_steps_per_s": rs / s, "engine_steps_per_s": steps / s, "seconds": s,
                         "configs": n_cfg, "requests_per_config": len(tr.n_in), "request_steps": rs,
                         "feasible_configs": int((sim["status"] == 0).sum().item()), "scheduler": "split-fuse",
                         # from rocprofv3 counters, not measured in this run (profiles/extra_kernels_valu_pmc.md)
                         "vector_issue_frac_profiled": counter_figure("simulate_vector_issue_frac")}
    a.record()
    ctx.simulate(gg, d_idx, d_rate, (tr.arrival_unit, tr.n_in, tr.n_out), sim, ws, scheduler=guide.SCHED_PREFILL_FIRST)
    b.record()
    torch.cuda.synchronize()
    s = a.elapsed_time(b) * 1e-3
    rs = int(sim["n_request_steps"].sum().item())
    extra["simulate_prefill_first"] = {"request_steps_per_s": rs / s, "seconds": s, "request_steps": rs,
                                       "engine_steps_per_s": int(sim["n_steps"].sum().item()) / s}
    # the same simulations with runs of decode-only steps advanced in closed form (same request-steps simulated)
    for name, sched in (("simulate_closed_form_runs", guide.SCHED_SPLIT_FUSE),
                        ("simulate_prefill_first_closed_form_runs", guide.SCHED_PREFILL_FIRST)):
        a.record()
        ctx.simulate(gg, d_idx, d_rate, (tr.arrival_unit, tr.n_in, tr.n_out), sim, ws,
                     scheduler=sched | guide.SIM_CLOSED_FORM_RUNS)
        b.record()
        torch.cuda.synchronize()
        s = a.elapsed_time(b) * 1e-3
        rs = int(sim["n_request_steps"].sum().item())
        extra[name] = {"request_steps_per_s": rs / s, "seconds": s, "request_steps": rs,
                       "engine_steps_per_s": int(sim["n_steps"].sum().item()) / s}
    return extra


def cpu_baseline(g, np, wl, host, selected, front):
    """The oracle as it stands, single thread, on 192 blocks of 1024 rows spread evenly over the grid; the rows the
    step selected (top-3 and front members) are re-evaluated by the oracle one by one."""
    from oracle import guide_oracle as ora
    og = ora.Grid(wl.models_array(g.models), wl.hw_array(g.hws), [a.array() for a in g.axes])
    blocks, rows = 192, 1024
    firsts = np.linspace(0, g.size - rows, blocks).astype(np.int64)
    ora.eval_grid(og, 0, 16)
    t0 = time.perf_counter()
    for f in firsts:
        ora.eval_grid(og, int(f), rows)
    dt_ = time.perf_counter() - t0
    # the serving simulation on the first 512 of the benchmark's 65 536 configurations
    idx, rate = wl.sim_configs(g, 65536)
    tr = wl.request_trace()
    t0 = time.perf_counter()
    sim = ora.simulate_grid(og, idx[:512], rate[:512], tr.arrival_unit, tr.n_in, tr.n_out)
    dt_sim = time.perf_counter() - t0
    worst = 0.0
    for row in list(selected) + [int(i) for i in front]:
        e = ora.eval_grid(og, int(row), 1)
        for k in ("t_prefill", "t_decode", "t_batch", "decode_tok_s", "cost"):
            worst = max(worst, abs(float(host[k][row]) - float(e[k][0])) / max(abs(float(e[k][0])), 1e-300))
        assert int(host["b_max"].view(np.uint32)[row]) == int(e["b_max"][0]) and int(host["feasible"][row]) == int(e["feasible"][0])
    return {"value": blocks * rows / dt_, "unit": "configs/s", "cores": 1, "kind": "oracle",
            "sample": f"{blocks} blocks of {rows} consecutive configurations spread evenly over the 1900800-row grid "
                      f"(eval_grid only), {dt_:.1f} s", "host_cores_available": os.cpu_count(),
            "simulate_request_steps_per_s": float(sim["n_request_steps"].sum()) / dt_sim,
            "simulate_sample": f"first 512 of the 65536 simulated configurations x 1024 requests, {dt_sim:.1f} s",
            "selected_rows_vs_oracle": {"rows": len(selected) + len(front), "max_rel_err": worst}}


if __name__ == "__main__":
    main()
