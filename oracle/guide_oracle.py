"""ctypes wrapper of the CPU oracle (oracle/guide_oracle.c).

TEST INFRASTRUCTURE: only tests, the smoke check and the benchmark's
CPU-baseline leg may import this.  It takes plain numpy arrays / Python numbers
and imports nothing from the GPU package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "guide_oracle.c")
_LIB = os.path.join(_HERE, "libguide_oracle.so")
GCC_FLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra", "-shared", "-fPIC"]

ROOFLINE, ADDITIVE = 0, 1
SIM_OK, SIM_INFEASIBLE = 0, 1
SCHED_SPLIT_FUSE, SCHED_PREFILL_FIRST = 0, 1
SIM_CLOSED_FORM_RUNS = 256        # OR-ed into the scheduler
NO_INDEX = 2 ** 64 - 1


# GUIDE_ORACLE_SANITIZE=1: an AddressSanitizer + UndefinedBehaviorSanitizer build (the process must then run with
# the sanitizer runtime preloaded: LD_PRELOAD=$(gcc -print-file-name=libasan.so)); errors abort the process.
SANITIZE = os.environ.get("GUIDE_ORACLE_SANITIZE") == "1"
if SANITIZE:
    _LIB = os.path.join(_HERE, "libguide_oracle_san.so")
    GCC_FLAGS = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                 "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra", "-shared", "-fPIC"]


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *GCC_FLAGS, "-o", _LIB, _SRC, "-lm"])
    return _LIB


class Model(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in ("L", "d", "n_h", "n_kv", "d_ff", "V", "E", "k")]


class Hw(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("peak", "bw", "cap", "link_bw", "link_lat")]


class Knobs(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("b", "s_in", "s_out", "p", "wbits", "blk", "mbt")]


class Metrics(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("t_prefill", "t_decode", "t_batch", "decode_tok_s", "cost", "tpot")] + \
               [("b_max", C.c_uint32), ("feasible", C.c_uint32)]


class GridC(C.Structure):
    _fields_ = [("models", C.POINTER(Model)), ("n_models", C.c_uint32),
                ("hws", C.POINTER(Hw)), ("n_hws", C.c_uint32),
                ("axis", C.POINTER(C.c_uint64) * 9), ("count", C.c_uint32 * 9)]


class SimOut(C.Structure):
    _fields_ = [("ttft_p50", C.c_double), ("ttft_p99", C.c_double), ("mean_tpot", C.c_double),
                ("tokens_s", C.c_double), ("status", C.c_uint32), ("n_steps", C.c_uint64),
                ("n_request_steps", C.c_uint64), ("min_admit_margin", C.c_double)]


class SpaceC(C.Structure):
    _fields_ = [("heads", C.POINTER(C.c_uint32)), ("peak", C.POINTER(C.c_double)), ("bw", C.POINTER(C.c_double)),
                ("cap", C.POINTER(C.c_double)), ("batch", C.POINTER(C.c_uint32)), ("s_in", C.POINTER(C.c_uint32)),
                ("s_out", C.POINTER(C.c_uint32)), ("tp", C.POINTER(C.c_uint32)), ("wbits", C.POINTER(C.c_uint32)),
                ("kv_block", C.POINTER(C.c_uint32)), ("mbt", C.POINTER(C.c_uint32)),
                ("kv_choices", C.POINTER(C.c_uint32)),
                ("layers_lo", C.c_uint32), ("layers_n", C.c_uint32), ("ffn_lo_x2", C.c_uint32),
                ("ffn_span_x2", C.c_uint32), ("vocab", C.c_uint32), ("link_div", C.c_double)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.ora_params_total.restype = C.c_double
        _lib.ora_params_layer_active.restype = C.c_double
        _lib.ora_pass.restype = C.c_double
        _lib.ora_pass.argtypes = [C.POINTER(Model), C.POINTER(Hw), C.c_double, C.c_double, C.c_uint64, C.c_uint64,
                                  C.c_int, C.c_double, C.c_double, C.c_double, C.c_double,
                                  C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        _lib.ora_weight_bytes_gpu.restype = C.c_double
        _lib.ora_weight_bytes_gpu.argtypes = [C.POINTER(Model), C.c_uint64, C.c_uint64]
        _lib.ora_kv_bytes_token.restype = C.c_double
        _lib.ora_kv_bytes_token.argtypes = [C.POINTER(Model), C.c_uint64]
        _lib.ora_prefill.restype = C.c_double
        _lib.ora_prefill.argtypes = [C.POINTER(Model), C.POINTER(Hw), C.POINTER(Knobs), C.c_double, C.c_double, C.c_int]
        _lib.ora_eval.argtypes = [C.POINTER(Model), C.POINTER(Hw), C.POINTER(Knobs), C.c_double, C.c_double, C.c_int,
                                  C.POINTER(Metrics)]
        _lib.ora_grid_size.restype = C.c_uint64
        _lib.ora_eval_grid.argtypes = [C.POINTER(GridC), C.c_uint64, C.c_uint64, C.c_double, C.c_double, C.c_int] + \
                                      [C.c_void_p] * 7
        _lib.ora_eval_extras_grid.argtypes = [C.POINTER(GridC), C.c_uint64, C.c_uint64, C.c_uint32, C.c_int,
                                              C.c_double] + [C.c_void_p] * 12
        _lib.ora_eval_sweep.argtypes = [C.POINTER(Model), C.POINTER(Hw), C.POINTER(Knobs), C.c_uint32,
                                        C.c_void_p, C.c_void_p, C.c_int, C.c_void_p,
                                        C.POINTER(C.c_double), C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
        _lib.ora_eval_sweep_grid.argtypes = [C.POINTER(GridC), C.c_uint64, C.c_uint64, C.c_uint32,
                                             C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                             C.c_void_p]
        _lib.ora_simulate.argtypes = [C.POINTER(Model), C.POINTER(Hw), C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint64,
                                      C.c_uint64, C.c_double, C.c_int, C.c_int, C.c_uint32, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.POINTER(SimOut), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        _lib.ora_decode_run_time.restype = C.c_double
        _lib.ora_decode_run_time.argtypes = [C.POINTER(Model), C.POINTER(Hw), C.c_uint64, C.c_uint64, C.c_int,
                                             C.c_double, C.c_double, C.c_double]
        _lib.ora_decode_run_steps.restype = C.c_double
        _lib.ora_decode_run_steps.argtypes = [C.POINTER(Model), C.POINTER(Hw), C.c_uint64, C.c_uint64, C.c_int,
                                              C.c_double, C.c_double, C.c_uint64]
        _lib.ora_simulate_grid.argtypes = [C.POINTER(GridC), C.c_void_p, C.c_void_p, C.c_uint32, C.c_int, C.c_int,
                                           C.c_uint32,
                                           C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        _lib.ora_select_topk.argtypes = [C.c_uint64, C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p]
        for f in (_lib.ora_pareto_brute, _lib.ora_pareto_sweep):
            f.restype = C.c_uint64
            f.argtypes = [C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64]
        _lib.ora_philox4x64_10.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        _lib.ora_sample_config.argtypes = [C.POINTER(SpaceC), C.c_uint64, C.c_uint64, C.POINTER(Model), C.POINTER(Hw),
                                           C.POINTER(Knobs)]
        _lib.ora_bucket.restype = C.c_uint32
        _lib.ora_bucket.argtypes = [C.c_double, C.c_void_p, C.c_uint32]
        _lib.ora_hist_bin.restype = C.c_uint32
        _lib.ora_hist_bin.argtypes = [C.c_double]
        _lib.ora_eval_sampled.argtypes = [C.POINTER(SpaceC), C.c_uint64, C.c_uint64, C.c_uint64, C.c_int,
                                          C.c_void_p, C.c_uint32, C.c_double] + [C.c_void_p] * 10
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def model(row) -> Model:
    return Model(*[int(v) for v in row])


def hw(row) -> Hw:
    return Hw(*[float(v) for v in row])


def knobs(b, s_in, s_out, p=1, wbits=16, blk=16, mbt=8192) -> Knobs:
    return Knobs(int(b), int(s_in), int(s_out), int(p), int(wbits), int(blk), int(mbt))


def params_total(m) -> float:
    return lib().ora_params_total(C.byref(m))


def params_layer_active(m) -> float:
    return lib().ora_params_layer_active(C.byref(m))


def pass_detail(m, h, p, wbits, T, Q, K, n_lm, e_c=1.0, e_b=1.0, time_model=ROOFLINE):
    F = np.zeros(8); B = np.zeros(8); t = np.zeros(8); ar = np.zeros(1)
    tp = lib().ora_pass(C.byref(m), C.byref(h), e_c, e_b, p, wbits, time_model, float(T), float(Q), float(K),
                        float(n_lm), _ptr(F), _ptr(B), _ptr(t), _ptr(ar))
    return dict(F=F, B=B, t=t, t_ar=float(ar[0]), t_pass=tp)


def weight_bytes_gpu(m, p, wbits) -> float:
    return lib().ora_weight_bytes_gpu(C.byref(m), p, wbits)


def kv_bytes_token(m, p) -> float:
    return lib().ora_kv_bytes_token(C.byref(m), p)


def memory(m, h, kn):
    kv = C.c_double(); ca = C.c_double(); fe = C.c_uint32(); bm = C.c_uint32()
    f = lib().ora_memory
    f.argtypes = [C.POINTER(Model), C.POINTER(Hw), C.POINTER(Knobs), C.POINTER(C.c_double), C.POINTER(C.c_double),
                  C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
    f(C.byref(m), C.byref(h), C.byref(kn), C.byref(kv), C.byref(ca), C.byref(fe), C.byref(bm))
    return dict(kv_req=kv.value, c_avail=ca.value, feasible=fe.value, b_max=bm.value)


def prefill(m, h, kn, e_c=1.0, e_b=1.0, time_model=ROOFLINE) -> float:
    return lib().ora_prefill(C.byref(m), C.byref(h), C.byref(kn), e_c, e_b, time_model)


def evaluate(m, h, kn, e_c=1.0, e_b=1.0, time_model=ROOFLINE) -> Metrics:
    r = Metrics()
    lib().ora_eval(C.byref(m), C.byref(h), C.byref(kn), e_c, e_b, time_model, C.byref(r))
    return r


class Grid:
    """Oracle-side grid: model rows (u32[n,8]), hardware rows (f64[n,5]) and nine
    explicit u64 value arrays (slow -> fast)."""

    def __init__(self, models_rows, hw_rows, axis_values):
        self._models = (Model * len(models_rows))(*[model(r) for r in models_rows])
        self._hws = (Hw * len(hw_rows))(*[hw(r) for r in hw_rows])
        self._axes = [np.ascontiguousarray(a, dtype=np.uint64) for a in axis_values]
        assert len(self._axes) == 9
        g = GridC()
        g.models = C.cast(self._models, C.POINTER(Model)); g.n_models = len(models_rows)
        g.hws = C.cast(self._hws, C.POINTER(Hw)); g.n_hws = len(hw_rows)
        for i, a in enumerate(self._axes):
            g.axis[i] = a.ctypes.data_as(C.POINTER(C.c_uint64))
            g.count[i] = len(a)
        self.c = g
        self.size = int(lib().ora_grid_size(C.byref(g)))


def eval_grid(g: Grid, first=0, count=None, e_c=1.0, e_b=1.0, time_model=ROOFLINE):
    count = g.size - first if count is None else count
    cols = {k: np.empty(count, dtype=np.float64) for k in ("t_prefill", "t_decode", "t_batch", "decode_tok_s", "cost")}
    cols["b_max"] = np.empty(count, dtype=np.uint32)
    cols["feasible"] = np.empty(count, dtype=np.uint8)
    rc = lib().ora_eval_grid(C.byref(g.c), first, count, e_c, e_b, time_model,
                             *[_ptr(cols[k]) for k in ("t_prefill", "t_decode", "t_batch", "decode_tok_s", "cost",
                                                        "b_max", "feasible")])
    if rc:
        raise ValueError("oracle: index outside the grid")
    return cols


def eval_extras_grid(g: Grid, n_gpus, first=0, count=None, time_model=ROOFLINE, kv_keep=1.0):
    count = g.size - first if count is None else count
    u32 = ("s_max", "dp_max", "b_adj", "n_sub_batches", "n_segments", "s_adj", "b_max_kept", "feasible_kept",
           "s_max_kept")
    out = {k: np.empty(count, dtype=np.uint32) for k in u32}
    out.update(max_parallelism=np.empty(count, dtype=np.uint64), cluster_tok_s=np.empty(count),
               paper_tok_s=np.empty(count))
    rc = lib().ora_eval_extras_grid(C.byref(g.c), first, count, n_gpus, time_model, float(kv_keep),
           *[_ptr(out[k]) for k in ("s_max", "dp_max", "max_parallelism", "cluster_tok_s", "paper_tok_s", "b_adj",
                                          "n_sub_batches", "n_segments", "s_adj", "b_max_kept", "feasible_kept",
                                          "s_max_kept")])
    if rc:
        raise ValueError("oracle: index outside the grid")
    return out


def eval_sweep_grid(g: Grid, e_c, e_b, first=0, count=None, time_model=ROOFLINE):
    count = g.size - first if count is None else count
    e_c = np.ascontiguousarray(e_c, dtype=np.float64); e_b = np.ascontiguousarray(e_b, dtype=np.float64)
    stats = np.empty((6, count), dtype=np.float64)
    cost = np.empty(count, dtype=np.float64); bm = np.empty(count, dtype=np.uint32); fe = np.empty(count, dtype=np.uint8)
    rc = lib().ora_eval_sweep_grid(C.byref(g.c), first, count, len(e_c), _ptr(e_c), _ptr(e_b), time_model,
                                   _ptr(stats), _ptr(cost), _ptr(bm), _ptr(fe))
    if rc:
        raise ValueError("oracle: index outside the grid")
    names = ("ttft_mean", "ttft_p10", "ttft_p90", "t_batch_mean", "t_batch_p10", "t_batch_p90")
    out = {n: stats[i] for i, n in enumerate(names)}
    out.update(cost=cost, b_max=bm, feasible=fe)
    return out


def simulate(m, h, p, wbits, blk, mbt, max_seqs, rate, arr_unit, n_in, n_out, time_model=ROOFLINE, detail=False,
             scheduler=SCHED_SPLIT_FUSE):
    arr_unit = np.ascontiguousarray(arr_unit, dtype=np.float64)
    n_in = np.ascontiguousarray(n_in, dtype=np.uint32); n_out = np.ascontiguousarray(n_out, dtype=np.uint32)
    n = len(arr_unit)
    o = SimOut()
    ttft = first = fin = None
    mf = C.c_int64(0)
    if detail:
        ttft = np.empty(n); first = np.empty(n); fin = np.empty(n)
    lib().ora_simulate(C.byref(m), C.byref(h), p, wbits, blk, mbt, max_seqs, float(rate), time_model, scheduler, n,
                       _ptr(arr_unit), _ptr(n_in), _ptr(n_out), C.byref(o), _ptr(ttft), _ptr(first), _ptr(fin),
                       C.cast(C.byref(mf), C.c_void_p))
    res = dict(ttft_p50=o.ttft_p50, ttft_p99=o.ttft_p99, mean_tpot=o.mean_tpot, tokens_s=o.tokens_s,
               status=o.status, n_steps=o.n_steps, n_request_steps=o.n_request_steps,
               min_admit_margin=o.min_admit_margin)
    if detail:
        res.update(ttft=ttft, first=first, fin=fin, min_free=mf.value)
    return res


def decode_run_time(m, h, p, wbits, T, C0, r, time_model=ROOFLINE) -> float:
    return lib().ora_decode_run_time(C.byref(m), C.byref(h), p, wbits, time_model, float(T), float(C0), float(r))


def decode_run_steps(m, h, p, wbits, T, C0, r, time_model=ROOFLINE) -> float:
    return lib().ora_decode_run_steps(C.byref(m), C.byref(h), p, wbits, time_model, float(T), float(C0), int(r))


def simulate_grid(g: Grid, cfg_idx, rate, arr_unit, n_in, n_out, time_model=ROOFLINE, scheduler=SCHED_SPLIT_FUSE):
    cfg_idx = np.ascontiguousarray(cfg_idx, dtype=np.uint32); rate = np.ascontiguousarray(rate, dtype=np.float64)
    arr_unit = np.ascontiguousarray(arr_unit, dtype=np.float64)
    n_in = np.ascontiguousarray(n_in, dtype=np.uint32); n_out = np.ascontiguousarray(n_out, dtype=np.uint32)
    outs = (SimOut * len(cfg_idx))()
    rc = lib().ora_simulate_grid(C.byref(g.c), _ptr(cfg_idx), _ptr(rate), len(cfg_idx), time_model, scheduler,
                                 len(arr_unit),
                                 _ptr(arr_unit), _ptr(n_in), _ptr(n_out), C.cast(outs, C.c_void_p))
    if rc:
        raise ValueError("oracle: index outside the grid")
    names = ("ttft_p50", "ttft_p99", "mean_tpot", "tokens_s", "min_admit_margin")
    res = {k: np.array([getattr(o, k) for o in outs], dtype=np.float64) for k in names}
    res["status"] = np.array([o.status for o in outs], dtype=np.uint32)
    res["n_steps"] = np.array([o.n_steps for o in outs], dtype=np.uint64)
    res["n_request_steps"] = np.array([o.n_request_steps for o in outs], dtype=np.uint64)
    return res


def select_topk(obj, feasible=None, constraints=(), group=None, n_groups=1, k=1):
    """constraints: sequence of (column, cap).  Returns idx[n_groups,k], val[n_groups,k], count[n_groups]."""
    obj = np.ascontiguousarray(obj, dtype=np.float64)
    n = len(obj)
    fe = None if feasible is None else np.ascontiguousarray(feasible, dtype=np.uint8)
    cols = [np.ascontiguousarray(c, dtype=np.float64) for c, _ in constraints]
    caps = np.array([cap for _, cap in constraints], dtype=np.float64)
    colp = (C.c_void_p * max(1, len(cols)))(*[c.ctypes.data for c in cols])
    gr = None if group is None else np.ascontiguousarray(group, dtype=np.uint32)
    idx = np.empty((n_groups, k), dtype=np.uint64); val = np.empty((n_groups, k), dtype=np.float64)
    cnt = np.empty(n_groups, dtype=np.uint64)
    lib().ora_select_topk(n, _ptr(obj), _ptr(fe), len(cols), C.cast(colp, C.c_void_p), _ptr(caps), _ptr(gr),
                          n_groups, k, _ptr(idx), _ptr(val), _ptr(cnt))
    return idx, val, cnt


def _pareto(fn, x, y, mask):
    x = np.ascontiguousarray(x, dtype=np.float64); y = np.ascontiguousarray(y, dtype=np.float64)
    mk = None if mask is None else np.ascontiguousarray(mask, dtype=np.uint8)
    out = np.empty(max(1, len(x)), dtype=np.uint64)
    nf = fn(len(x), _ptr(x), _ptr(y), _ptr(mk), _ptr(out), len(out))
    return out[:nf].copy()


def pareto_brute(x, y, mask=None):
    return _pareto(lib().ora_pareto_brute, x, y, mask)


def pareto_sweep(x, y, mask=None):
    return _pareto(lib().ora_pareto_sweep, x, y, mask)


def philox4x64_10(ctr, key):
    ctr = np.ascontiguousarray(ctr, dtype=np.uint64); key = np.ascontiguousarray(key, dtype=np.uint64)
    out = np.empty(4, dtype=np.uint64)
    lib().ora_philox4x64_10(_ptr(ctr), _ptr(key), _ptr(out))
    return out


class Space:
    """Oracle-side tables of the sampled space (plain arrays in, kept alive here)."""
    FIELDS = ("heads", "peak", "bw", "cap", "batch", "s_in", "s_out", "tp", "wbits", "kv_block", "mbt", "kv_choices")

    def __init__(self, **kw):
        self._keep = {}
        s = SpaceC()
        for f in self.FIELDS:
            dt = np.float64 if f in ("peak", "bw", "cap") else np.uint32
            a = np.ascontiguousarray(kw[f], dtype=dt)
            self._keep[f] = a
            setattr(s, f, a.ctypes.data_as(C.POINTER(C.c_double if dt == np.float64 else C.c_uint32)))
        for f in ("layers_lo", "layers_n", "ffn_lo_x2", "ffn_span_x2", "vocab"):
            setattr(s, f, int(kw[f]))
        s.link_div = float(kw["link_div"])
        self.c = s


def sample_config(sp: Space, seed, idx):
    m = Model(); h = Hw(); kn = Knobs()
    lib().ora_sample_config(C.byref(sp.c), seed, idx, C.byref(m), C.byref(h), C.byref(kn))
    return m, h, kn


def bucket(p_total, edges) -> int:
    e = np.ascontiguousarray(edges, dtype=np.float64)
    return lib().ora_bucket(float(p_total), _ptr(e), len(e))


def hist_bin(t) -> int:
    return lib().ora_hist_bin(float(t))


def eval_sampled(sp: Space, seed, first, count, edges, ttft_cap, time_model=ROOFLINE, columns=False):
    e = np.ascontiguousarray(edges, dtype=np.float64)
    nb = len(e) + 1
    fc = np.zeros(1, dtype=np.uint64); wv = np.empty(nb); wi = np.empty(nb, dtype=np.uint64)
    hist = np.zeros(256, dtype=np.uint64)
    cols = {}
    if columns:
        cols = dict(t_prefill=np.empty(count), t_batch=np.empty(count), cost=np.empty(count),
                    b_max=np.empty(count, dtype=np.uint32), feasible=np.empty(count, dtype=np.uint8),
                    bucket=np.empty(count, dtype=np.uint32))
    lib().ora_eval_sampled(C.byref(sp.c), seed, first, count, time_model, _ptr(e), len(e), float(ttft_cap),
                           _ptr(fc), _ptr(wv), _ptr(wi), _ptr(hist),
                           *[_ptr(cols.get(k)) for k in ("t_prefill", "t_batch", "cost", "b_max", "feasible", "bucket")])
    res = dict(feasible_count=int(fc[0]), win_val=wv, win_idx=wi, hist=hist)
    res.update(cols)
    return res
