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
