"""Test-side glue: turns the shared synthetic inputs into oracle objects.
(Tests may import both sides; the two sides never import each other.)"""
import numpy as np

from oracle import guide_oracle as go
from paper_2412_04788_amd import workloads as wl


def ora_grid(grid: wl.Grid) -> go.Grid:
    return go.Grid(wl.models_array(grid.models), wl.hw_array(grid.hws), [a.array() for a in grid.axes])


def ora_space(sp: wl.SampleSpace) -> go.Space:
    kw = {f: getattr(sp, f) for f in go.Space.FIELDS}
    kw.update(layers_lo=sp.layers_lo, layers_n=sp.layers_n, ffn_lo_x2=sp.ffn_lo_x2, ffn_span_x2=sp.ffn_span_x2,
              vocab=sp.vocab, link_div=sp.link_div)
    return go.Space(**kw)


def ora_model(m: wl.Model) -> go.Model:
    return go.model(m.as_row())


def ora_hw(h: wl.Hardware) -> go.Hw:
    return go.hw(h.as_row())


def rel_err(a, b):
    a = np.asarray(a, dtype=np.float64); b = np.asarray(b, dtype=np.float64)
    den = np.maximum(np.abs(b), np.finfo(np.float64).tiny)
    with np.errstate(invalid="ignore"):
        e = np.abs(a - b) / den
    both_inf = np.isinf(a) & np.isinf(b) & (np.sign(a) == np.sign(b))
    e[both_inf] = 0.0
    e[(a == 0) & (b == 0)] = 0.0
    return e


# ------------------------------------------------------------- GPU-side glue

def gpu_grid(grid: wl.Grid):
    from paper_2412_04788_amd import guide
    return guide.GridArg([(a.values, a.geom2_start) for a in grid.axes])


def gpu_context(grid: wl.Grid):
    from paper_2412_04788_amd import guide
    ctx = guide.Context(0)
    ctx.set_models(wl.models_array(grid.models))
    ctx.set_hardware(wl.hw_array(grid.hws))
    return ctx


def gpu_space(sp: wl.SampleSpace) -> dict:
    d = {f: getattr(sp, f) for f in ("heads", "peak", "bw", "cap", "batch", "s_in", "s_out", "tp", "wbits",
                                      "kv_block", "mbt", "kv_choices")}
    d.update(layers_lo=sp.layers_lo, layers_n=sp.layers_n, ffn_lo_x2=sp.ffn_lo_x2, ffn_span_x2=sp.ffn_span_x2,
             vocab=sp.vocab, link_div=sp.link_div)
    return d


def metric_buffers(n, names=("t_prefill", "t_decode", "t_batch", "decode_tok_s", "cost", "b_max", "feasible")):
    import torch
    dt = {"b_max": torch.int32, "feasible": torch.uint8, "bucket": torch.int32}
    return {k: torch.empty(n, dtype=dt.get(k, torch.float64), device="cuda") for k in names}


def to_np(t, dtype=None):
    a = t.cpu().numpy()
    if dtype is not None:
        a = a.view(dtype)
    return a


# --------------------------------------------- the oracle on all host cores

def host_workers() -> int:
    """Threads for oracle sweeps: the oracle's C entry points hold no global state and ctypes releases the
    interpreter lock during a call, so independent ranges run side by side (at most 16 threads)."""
    import os
    return max(1, min(16, os.cpu_count() or 1))


def _chunks(total, chunk):
    return [(a, min(chunk, total - a)) for a in range(0, total, chunk)]


def ora_eval_grid_all(og: go.Grid, first=0, count=None, chunk=4096, **kw):
    """go.eval_grid over [first, first + count), ranges spread over the host cores."""
    from concurrent.futures import ThreadPoolExecutor
    count = og.size - first if count is None else count
    parts = _chunks(count, chunk)
    with ThreadPoolExecutor(host_workers()) as ex:
        res = list(ex.map(lambda p: go.eval_grid(og, first + p[0], p[1], **kw), parts))
    return {k: np.concatenate([r[k] for r in res]) for k in res[0]}


def ora_eval_sweep_grid_rows(og: go.Grid, e_c, e_b, starts, length, **kw):
    """go.eval_sweep_grid on the ranges [s, s + length) for s in starts; columns concatenated in that order."""
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(host_workers()) as ex:
        res = list(ex.map(lambda s: go.eval_sweep_grid(og, e_c, e_b, int(s), length, **kw), starts))
    return {k: np.concatenate([r[k] for r in res]) for k in res[0]}


def ora_simulate_grid_all(og: go.Grid, cfg_idx, rate, trace, chunk=32, **kw):
    from concurrent.futures import ThreadPoolExecutor
    parts = _chunks(len(cfg_idx), chunk)
    with ThreadPoolExecutor(host_workers()) as ex:
        res = list(ex.map(lambda p: go.simulate_grid(og, cfg_idx[p[0]:p[0] + p[1]], rate[p[0]:p[0] + p[1]],
                                                     trace.arrival_unit, trace.n_in, trace.n_out, **kw), parts))
    return {k: np.concatenate([r[k] for r in res]) for k in res[0]}


def ora_eval_sampled_all(osp: go.Space, seed, first, count, edges, ttft_cap, chunk=1 << 14, columns=True):
    """go.eval_sampled over a long range: per-range results merged in ascending order (sums; a bucket's winner is
    the first range's unless a later one is strictly cheaper, which keeps the lowest index on ties)."""
    from concurrent.futures import ThreadPoolExecutor
    parts = _chunks(count, chunk)
    with ThreadPoolExecutor(host_workers()) as ex:
        res = list(ex.map(lambda p: go.eval_sampled(osp, seed, first + p[0], p[1], edges, ttft_cap, columns=columns),
                          parts))
    out = dict(feasible_count=sum(r["feasible_count"] for r in res), hist=sum(r["hist"] for r in res),
               win_val=res[0]["win_val"].copy(), win_idx=res[0]["win_idx"].copy())
    for r in res[1:]:
        better = r["win_val"] < out["win_val"]
        out["win_val"][better] = r["win_val"][better]
        out["win_idx"][better] = r["win_idx"][better]
    if columns:
        for k in ("t_prefill", "t_batch", "cost", "b_max", "feasible", "bucket"):
            out[k] = np.concatenate([r[k] for r in res])
    return out
