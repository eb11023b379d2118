"""Thin ctypes binding of libguide.so (include/guide.h): argument marshalling
only.  Every step of the evaluated path runs in the HIP kernels; there is no
CPU fallback, and a missing library is an error.  Device buffers are torch
tensors (torch is used for device memory and streams only).
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libguide.so")

OK, E_ARG, E_RANGE, E_NOMEM, E_DEVICE = 0, -1, -2, -3, -4
TIME_ROOFLINE, TIME_ADDITIVE = 0, 1
AXIS_GEOM2, AXIS_TABLE = 0, 1
SELECT_TOPK, SELECT_PARETO = 0, 1
SIM_OK, SIM_INFEASIBLE, SIM_BAD_INPUT, SIM_INTERNAL = 0, 1, 2, 3
SCHED_SPLIT_FUSE, SCHED_PREFILL_FIRST = 0, 1
SIM_CLOSED_FORM_RUNS = 256       # OR-ed into simulate()'s scheduler
NO_INDEX = 2 ** 64 - 1
MAX_CONSTRAINTS = 4
STATIC_SELECT_MAX_ROWS = 1 << 21

EXPORTS = ("guide_create", "guide_destroy", "guide_last_error", "guide_set_models", "guide_set_hardware",
           "guide_eval_grid", "guide_eval_extras", "guide_eval_sampled", "guide_simulate_workspace_bytes", "guide_simulate",
           "guide_select_workspace_bytes", "guide_select", "guide_select_static",
           "guide_eval_select_workspace_bytes", "guide_eval_select",
           "guide_profile_enable", "guide_profile_read")


class GuideError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libguide error {code}: {msg}")
        self.code = code


class CModel(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in ("L", "d", "n_h", "n_kv", "d_ff", "V", "E", "k")]


class CHw(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("peak_flops", "hbm_bw", "cap_bytes", "link_bw", "link_lat")]


class CAxis(C.Structure):
    _fields_ = [("count", C.c_uint32), ("kind", C.c_uint32), ("start", C.c_uint64), ("values", C.POINTER(C.c_uint64))]


class CGrid(C.Structure):
    _fields_ = [(n, CAxis) for n in ("model", "hw", "batch", "s_in", "s_out", "tp", "wbits", "kv_block", "mbt")]


class CEff(C.Structure):
    _fields_ = [("n", C.c_uint32), ("e_c", C.c_void_p), ("e_b", C.c_void_p)]


METRIC_COLUMNS = ("t_prefill", "t_decode", "t_batch", "decode_tok_s", "cost", "b_max", "feasible")
STATS_COLUMNS = ("ttft_mean", "ttft_p10", "ttft_p90", "t_batch_mean", "t_batch_p10", "t_batch_p90", "cost", "b_max",
                 "feasible")
EXTRAS_COLUMNS = ("s_max", "dp_max", "max_parallelism", "cluster_tok_s", "paper_tok_s", "b_adj", "n_sub_batches",
                  "n_segments", "s_adj", "b_max_kept", "s_max_kept", "feasible_kept")
SAMPLED_COLUMNS = ("feasible_count", "win_val", "win_idx", "hist", "t_prefill", "t_batch", "cost", "b_max",
                   "feasible", "bucket")
SIM_COLUMNS = ("ttft_p50", "ttft_p99", "mean_tpot", "tokens_s", "status", "n_steps", "n_request_steps")


class CMetrics(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in METRIC_COLUMNS]


class CStats(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in STATS_COLUMNS]


class CExtras(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in EXTRAS_COLUMNS[:9]] + [("kv_keep", C.c_double)] + \
               [(n, C.c_void_p) for n in EXTRAS_COLUMNS[9:]]


class CSpace(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("heads", "peak", "bw", "cap", "batch", "s_in", "s_out", "tp", "wbits",
                                          "kv_block", "mbt", "kv_choices")] + \
               [(n, C.c_uint32) for n in ("layers_lo", "layers_n", "ffn_lo_x2", "ffn_span_x2", "vocab")] + \
               [("link_div", C.c_double)]


class CSampledOut(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in SAMPLED_COLUMNS]


class CTrace(C.Structure):
    _fields_ = [("n", C.c_uint32), ("arrival_unit", C.c_void_p), ("n_in", C.c_void_p), ("n_out", C.c_void_p)]


class CSimOut(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in SIM_COLUMNS]


class CConstraint(C.Structure):
    _fields_ = [("column", C.c_void_p), ("cap", C.c_double)]


class CSelectSpec(C.Structure):
    _fields_ = [("mode", C.c_uint32), ("objective", C.c_void_p), ("objective_y", C.c_void_p),
                ("feasible", C.c_void_p), ("n_constraints", C.c_uint32),
                ("constraints", CConstraint * MAX_CONSTRAINTS), ("group", C.c_void_p),
                ("n_groups", C.c_uint32), ("k", C.c_uint32)]


class CSelectOut(C.Structure):
    _fields_ = [("idx", C.c_void_p), ("val", C.c_void_p), ("count", C.c_void_p), ("capacity", C.c_uint64)]


COLUMN_IDS = {"t_prefill": 0, "t_decode": 1, "t_batch": 2, "decode_tok_s": 3, "cost": 4}


class CColumnConstraint(C.Structure):
    _fields_ = [("column", C.c_uint32), ("reserved", C.c_uint32), ("cap", C.c_double)]


class CColumnSelect(C.Structure):
    _fields_ = [("mode", C.c_uint32), ("objective", C.c_uint32), ("objective_y", C.c_uint32),
                ("use_feasible", C.c_uint32), ("n_constraints", C.c_uint32), ("k", C.c_uint32),
                ("constraints", CColumnConstraint * MAX_CONSTRAINTS), ("out", CSelectOut)]


_lib = None


def load() -> C.CDLL:
    """Loads libguide.so; raises if it has not been built (python -m paper_2412_04788_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: build it with paper_2412_04788_amd/build.py")
        # torch ships its own HIP runtime; it must be in the process before libguide's
        # dependency on libamdhip64 is resolved, or two runtimes would be loaded
        import torch  # noqa: F401
        lib = C.CDLL(LIB_PATH)
        lib.guide_create.argtypes = [C.POINTER(C.c_void_p), C.c_int]
        lib.guide_destroy.argtypes = [C.c_void_p]
        lib.guide_destroy.restype = None
        lib.guide_last_error.argtypes = [C.c_void_p]
        lib.guide_last_error.restype = C.c_char_p
        lib.guide_set_models.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32]
        lib.guide_set_hardware.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32]
        lib.guide_eval_grid.argtypes = [C.c_void_p, C.POINTER(CGrid), C.c_uint64, C.c_uint64, C.POINTER(CEff),
                                        C.c_uint32, C.POINTER(CMetrics), C.POINTER(CStats), C.c_void_p]
        lib.guide_eval_extras.argtypes = [C.c_void_p, C.POINTER(CGrid), C.c_uint64, C.c_uint64, C.c_uint32,
                                          C.c_uint32, C.POINTER(CExtras), C.c_void_p]
        lib.guide_eval_sampled.argtypes = [C.c_void_p, C.POINTER(CSpace), C.c_uint64, C.c_uint64, C.c_uint64,
                                           C.c_void_p, C.c_uint32, C.c_double, C.c_uint32, C.POINTER(CSampledOut),
                                           C.c_void_p]
        lib.guide_simulate_workspace_bytes.argtypes = [C.c_uint32, C.c_uint32]
        lib.guide_simulate_workspace_bytes.restype = C.c_size_t
        lib.guide_simulate.argtypes = [C.c_void_p, C.POINTER(CGrid), C.c_void_p, C.c_void_p, C.c_uint32,
                                       C.POINTER(CTrace), C.c_uint32, C.c_uint32, C.POINTER(CSimOut), C.c_void_p,
                                       C.c_size_t, C.c_void_p]
        lib.guide_select_workspace_bytes.argtypes = [C.POINTER(CSelectSpec), C.c_uint64]
        lib.guide_select_workspace_bytes.restype = C.c_size_t
        lib.guide_select.argtypes = [C.c_void_p, C.POINTER(CSelectSpec), C.c_uint64, C.POINTER(CSelectOut),
                                     C.c_void_p, C.c_size_t, C.c_void_p]
        lib.guide_select_static.argtypes = [C.c_void_p, C.POINTER(CSelectSpec), C.c_uint64, C.POINTER(CSelectOut),
                                            C.c_void_p]
        lib.guide_eval_select_workspace_bytes.argtypes = [C.c_void_p, C.c_uint32, C.c_uint64]
        lib.guide_eval_select_workspace_bytes.restype = C.c_size_t
        lib.guide_eval_select.argtypes = [C.c_void_p, C.POINTER(CGrid), C.c_uint64, C.c_uint64, C.POINTER(CEff),
                                          C.c_uint32, C.POINTER(CMetrics), C.c_void_p, C.c_uint32, C.c_void_p,
                                          C.c_size_t, C.c_void_p]
        lib.guide_profile_enable.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32]
        lib.guide_profile_read.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_uint32)]
        _lib = lib
    return _lib


class _Ref:
    """byref() of a ctypes struct that also keeps the struct (and what it points to) alive."""

    def __init__(self, struct, keep=None):
        self.struct, self.keep = struct, keep
        self._as_parameter_ = C.byref(struct)


class _Arr:
    """Address of a ctypes array, kept alive together with what its elements point to."""

    def __init__(self, arr, keep=None):
        self.arr, self.keep = arr, keep
        self._as_parameter_ = C.cast(arr, C.c_void_p)


class _Ptr:
    """Address of a host numpy array, kept alive."""

    def __init__(self, array):
        self.array = array
        self._as_parameter_ = C.c_void_p(array.ctypes.data)


def _dev_ptr(t) -> Optional[int]:
    """data_ptr() of a contiguous CUDA tensor (None passes NULL)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("device buffers must be contiguous CUDA tensors")
    return t.data_ptr()


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def make_axis(values: Sequence[int], geom2_start: int = 0):
    """Returns (CAxis, keep-alive array)."""
    ax = CAxis()
    ax.count = len(values)
    if geom2_start:
        ax.kind, ax.start, keep = AXIS_GEOM2, geom2_start, None
    else:
        keep = np.ascontiguousarray(values, dtype=np.uint64)
        ax.kind, ax.start = AXIS_TABLE, 0
        ax.values = keep.ctypes.data_as(C.POINTER(C.c_uint64))
    return ax, keep


class GridArg:
    """C grid descriptor from nine (values, geom2_start) pairs, slow -> fast."""

    def __init__(self, axes):
        assert len(axes) == 9
        self.c = CGrid()
        self._keep = []
        self.size = 1
        for (name, _), (values, start) in zip(CGrid._fields_, axes):
            ax, keep = make_axis(values, start)
            setattr(self.c, name, ax)
            self._keep.append(keep)
            self.size *= len(values)


class Context:
    """guide_ctx handle.  Methods mirror the C entry points one to one."""

    def __init__(self, device: int = 0):
        self._lib = load()
        h = C.c_void_p()
        rc = self._lib.guide_create(C.byref(h), device)
        if rc:
            raise GuideError(rc, "guide_create failed")
        self._h = h
        self.device = device

    def close(self):
        if getattr(self, "_h", None):
            self._lib.guide_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def last_error(self) -> str:
        return self._lib.guide_last_error(self._h).decode()

    def _check(self, rc):
        if rc:
            raise GuideError(rc, self.last_error())

    def set_models(self, rows):
        a = np.ascontiguousarray(rows, dtype=np.uint32).reshape(-1, 8)
        self._check(self._lib.guide_set_models(self._h, a.ctypes.data, len(a)))

    def set_hardware(self, rows):
        a = np.ascontiguousarray(rows, dtype=np.float64).reshape(-1, 5)
        self._check(self._lib.guide_set_hardware(self._h, a.ctypes.data, len(a)))

    def prepared(self, method: str, *args, **kw):
        """Marshals the arguments of `method` once and returns a zero-argument callable that
        repeats the same C call (for loops that re-issue one call many times; the stream is
        the one current at preparation time)."""
        calls = []
        real = self._invoke
        self._invoke = lambda fn, *a: calls.append((fn, a))
        try:
            getattr(self, method)(*args, **kw)
        finally:
            self._invoke = real
        (fn, a), = calls
        keep = (args, kw)

        def run(_fn=fn, _a=a, _keep=keep, _check=self._check):
            _check(_fn(*_a))
        return run

    def _invoke(self, fn, *a):
        self._check(fn(*a))

    def eval_grid(self, grid: GridArg, first: int, count: int, out: dict = None, stats: dict = None,
                  e_c=None, e_b=None, time_model: int = TIME_ROOFLINE, stream=None):
        """out / stats: dicts column name -> CUDA tensor (missing = not written)."""
        eff = None
        if e_c is not None:
            e_c = np.ascontiguousarray(e_c, dtype=np.float64)
            e_b = np.ascontiguousarray(e_b, dtype=np.float64)
            eff = CEff(len(e_c), e_c.ctypes.data, e_b.ctypes.data)
        cm = cs = None
        if out is not None:
            cm = CMetrics(*[_dev_ptr(out.get(k)) for k in METRIC_COLUMNS])
        if stats is not None:
            cs = CStats(*[_dev_ptr(stats.get(k)) for k in STATS_COLUMNS])
        self._invoke(self._lib.guide_eval_grid, self._h, _Ref(grid.c, grid), first, count,
                     _Ref(eff, (e_c, e_b)) if eff else None, time_model,
                     _Ref(cm) if cm else None, _Ref(cs) if cs else None, _stream_ptr(stream))

    @staticmethod
    def column_select(mode: int, objective: str, out_idx, out_val, out_count, objective_y: str = None,
                      use_feasible: bool = True, constraints=(), k: int = 1, capacity: int = 0) -> CColumnSelect:
        """guide_column_select from column names; constraints = [(column name, cap), ...]."""
        c = CColumnSelect()
        c.mode = mode
        c.objective = COLUMN_IDS[objective]
        c.objective_y = COLUMN_IDS[objective_y] if objective_y is not None else 0
        c.use_feasible = 1 if use_feasible else 0
        c.n_constraints = len(constraints)
        for i, (col, cap) in enumerate(list(constraints)[:MAX_CONSTRAINTS]):
            c.constraints[i].column = COLUMN_IDS[col]
            c.constraints[i].cap = float(cap)
        c.k = k
        c.out = CSelectOut(_dev_ptr(out_idx), _dev_ptr(out_val), _dev_ptr(out_count), capacity)
        c._keep = (out_idx, out_val, out_count)
        return c

    def eval_select_workspace_bytes(self, selections: Sequence[CColumnSelect], count: int) -> int:
        arr = (CColumnSelect * max(len(selections), 1))(*selections)
        return self._lib.guide_eval_select_workspace_bytes(C.cast(arr, C.c_void_p), len(selections), count)

    def eval_select(self, grid: GridArg, first: int, count: int, out: dict, selections: Sequence[CColumnSelect],
                    workspace, e_c=None, e_b=None, time_model: int = TIME_ROOFLINE, stream=None):
        """guide_eval_select: evaluate [first, first + count) into `out` and run the selections on it."""
        eff = None
        if e_c is not None:
            e_c = np.ascontiguousarray([e_c], dtype=np.float64).reshape(-1)
            e_b = np.ascontiguousarray([e_b], dtype=np.float64).reshape(-1)
            eff = CEff(len(e_c), e_c.ctypes.data, e_b.ctypes.data)
        cm = CMetrics(*[_dev_ptr(out.get(k)) for k in METRIC_COLUMNS])
        arr = (CColumnSelect * max(len(selections), 1))(*selections)
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        self._invoke(self._lib.guide_eval_select, self._h, _Ref(grid.c, grid), first, count,
                     _Ref(eff, (e_c, e_b)) if eff else None, time_model, _Ref(cm, out),
                     _Arr(arr, selections), len(selections),
                     _dev_ptr(workspace), ws_bytes, _stream_ptr(stream))

    def profile_enable(self, capacity: int, every: int = 1):
        self._check(self._lib.guide_profile_enable(self._h, capacity, every))

    def profile_read(self, capacity: int) -> np.ndarray:
        """Elapsed milliseconds of the evaluation kernels timed since the last read."""
        ms = np.zeros(max(capacity, 1), dtype=np.float32)
        n = C.c_uint32(0)
        self._check(self._lib.guide_profile_read(self._h, ms.ctypes.data, C.byref(n)))
        return ms[:n.value].copy()

    def eval_extras(self, grid: GridArg, first: int, count: int, n_gpus: int, out: dict,
                    time_model: int = TIME_ROOFLINE, stream=None, kv_keep: float = 0.0):
        ce = CExtras(**{k: _dev_ptr(out.get(k)) for k in EXTRAS_COLUMNS}, kv_keep=float(kv_keep))
        self._invoke(self._lib.guide_eval_extras, self._h, _Ref(grid.c, grid), first, count, n_gpus, time_model,
                     _Ref(ce), _stream_ptr(stream))

    def eval_sampled(self, space: dict, seed: int, first: int, count: int, edges, ttft_cap: float, out: dict,
                     time_model: int = TIME_ROOFLINE, stream=None):
        """space: dict of host numpy tables and scalars named as guide_space's fields."""
        keep = {}
        cs = CSpace()
        for name in ("heads", "batch", "s_in", "s_out", "tp", "wbits", "kv_block", "mbt", "kv_choices"):
            keep[name] = np.ascontiguousarray(space[name], dtype=np.uint32)
            setattr(cs, name, keep[name].ctypes.data)
        for name in ("peak", "bw", "cap"):
            keep[name] = np.ascontiguousarray(space[name], dtype=np.float64)
            setattr(cs, name, keep[name].ctypes.data)
        for name in ("layers_lo", "layers_n", "ffn_lo_x2", "ffn_span_x2", "vocab"):
            setattr(cs, name, int(space[name]))
        cs.link_div = float(space["link_div"])
        edges = np.ascontiguousarray(edges, dtype=np.float64)
        co = CSampledOut(*[_dev_ptr(out.get(k)) for k in SAMPLED_COLUMNS])
        self._invoke(self._lib.guide_eval_sampled, self._h, _Ref(cs, keep), seed, first, count,
                     _Ptr(edges), len(edges), ttft_cap, time_model, _Ref(co), _stream_ptr(stream))

    def simulate_workspace_bytes(self, n_cfg: int, n_requests: int) -> int:
        return self._lib.guide_simulate_workspace_bytes(n_cfg, n_requests)

    def simulate(self, grid: GridArg, cfg_idx, rate, trace, out: dict, workspace, time_model: int = TIME_ROOFLINE,
                 scheduler: int = SCHED_SPLIT_FUSE, stream=None):
        """cfg_idx (u32) / rate (f64): CUDA tensors; trace: (arrival_unit, n_in, n_out) host arrays."""
        arr = np.ascontiguousarray(trace[0], dtype=np.float64)
        n_in = np.ascontiguousarray(trace[1], dtype=np.uint32)
        n_out = np.ascontiguousarray(trace[2], dtype=np.uint32)
        ct = CTrace(len(arr), arr.ctypes.data, n_in.ctypes.data, n_out.ctypes.data)
        co = CSimOut(*[_dev_ptr(out.get(k)) for k in SIM_COLUMNS])
        self._invoke(self._lib.guide_simulate, self._h, _Ref(grid.c, grid), _dev_ptr(cfg_idx), _dev_ptr(rate),
                     cfg_idx.numel(), _Ref(ct, (arr, n_in, n_out)), time_model, scheduler, _Ref(co),
                     _dev_ptr(workspace), workspace.numel() * workspace.element_size(), _stream_ptr(stream))

    def _select_spec(self, mode, objective, objective_y, feasible, constraints, group, n_groups, k):
        s = CSelectSpec()
        s.mode = mode
        s.objective = _dev_ptr(objective)
        s.objective_y = _dev_ptr(objective_y)
        s.feasible = _dev_ptr(feasible)
        s.n_constraints = len(constraints)
        for i, (col, cap) in enumerate(constraints[:MAX_CONSTRAINTS]):
            s.constraints[i].column = _dev_ptr(col)
            s.constraints[i].cap = float(cap)
        s.group = _dev_ptr(group)
        s.n_groups = n_groups
        s.k = k
        return s

    def select_workspace_bytes(self, mode: int, n: int, n_groups: int = 1) -> int:
        s = CSelectSpec()
        s.mode, s.n_groups, s.k = mode, n_groups, 1
        return self._lib.guide_select_workspace_bytes(C.byref(s), n)

    def select(self, mode: int, n: int, objective, out_idx, out_val, out_count, workspace, objective_y=None,
               feasible=None, constraints=(), group=None, n_groups: int = 1, k: int = 1, capacity: int = 0,
               stream=None):
        s = self._select_spec(mode, objective, objective_y, feasible, list(constraints), group, n_groups, k)
        o = CSelectOut(_dev_ptr(out_idx), _dev_ptr(out_val), _dev_ptr(out_count), capacity)
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        self._invoke(self._lib.guide_select, self._h, _Ref(s), n, _Ref(o), _dev_ptr(workspace), ws_bytes,
                     _stream_ptr(stream))

    def select_static(self, mode: int, n: int, objective, out_idx, out_val, out_count, objective_y=None,
                      feasible=None, constraints=(), group=None, n_groups: int = 1, k: int = 1, capacity: int = 0,
                      stream=None):
        """guide_select_static: guide_select on the library's static device scratch (no workspace, no allocation)."""
        s = self._select_spec(mode, objective, objective_y, feasible, list(constraints), group, n_groups, k)
        o = CSelectOut(_dev_ptr(out_idx), _dev_ptr(out_val), _dev_ptr(out_count), capacity)
        self._invoke(self._lib.guide_select_static, self._h, _Ref(s), n, _Ref(o), _stream_ptr(stream))
