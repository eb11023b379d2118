"""Seeded synthetic inputs for the GUIDE deployment-optimiser hot path.

This module only *describes inputs*: model shapes, hardware profiles, grid axes,
efficiency samples, request traces and lattices.  It holds none of the
performance model's arithmetic and imports neither the CPU oracle nor the HIP
binding; both are fed from here so that they see bit-identical inputs.

The paper evaluates on its own measurements of four public checkpoints
(Experiments, "Experimental Setup"); none of that data is needed here.  The
five workloads below stand in for its sweep (batch {4..32} x prompt
{128..1024} x 256 generated tokens), which is a 16-point subset of the
tiny grid's axes.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence

import numpy as np

GIB = float(2 ** 30)
N_REQ = 1024            # requests per simulated trace
N_LATTICE = 1024        # points per log-uniform lattice of the sampled space
SEED = 20241204

AXIS_NAMES = ("model", "hw", "batch", "s_in", "s_out", "tp", "wbits", "kv_block", "mbt")


@dataclass(frozen=True)
class Model:
    """Decoder architecture (Model Analyzer inputs: layers N, hidden H, ...)."""
    name: str
    L: int
    d: int
    n_h: int
    n_kv: int
    d_ff: int
    V: int = 32000
    E: int = 1
    k: int = 1

    def as_row(self):
        return (self.L, self.d, self.n_h, self.n_kv, self.d_ff, self.V, self.E, self.k)


@dataclass(frozen=True)
class Hardware:
    """Pre-registered GPU record: compute perf, memory BW, capacity, comm BW, latency."""
    peak_flops: float
    hbm_bw: float
    cap_bytes: float
    link_bw: float
    link_lat: float = 0.0

    def as_row(self):
        return (self.peak_flops, self.hbm_bw, self.cap_bytes, self.link_bw, self.link_lat)


# Public architecture shapes (layers, hidden, heads, kv heads, ffn).
DENSE_7B = Model("dense-7b", 32, 4096, 32, 32, 11008)
DENSE_13B = Model("dense-13b", 40, 5120, 40, 40, 13824)
DENSE_34B = Model("dense-34b-gqa", 48, 8192, 64, 8, 22016)
DENSE_70B = Model("dense-70b-gqa", 80, 8192, 64, 8, 28672)
MOE_8X = Model("moe-8x-top2", 32, 4096, 32, 8, 14336, E=8, k=2)
MODELS_FULL = (DENSE_7B, DENSE_13B, DENSE_34B, DENSE_70B, MOE_8X)

HW_TINY = Hardware(1.0e15, 5.0e12, 192 * GIB, 4.0e11, 0.0)


def models_array(models: Sequence[Model]) -> np.ndarray:
    return np.ascontiguousarray([m.as_row() for m in models], dtype=np.uint32)


def hw_array(hws: Sequence[Hardware]) -> np.ndarray:
    return np.ascontiguousarray([h.as_row() for h in hws], dtype=np.float64)


def hw_profiles(seed: int = SEED, n: int = 6) -> List[Hardware]:
    """Six profiles: peak log-uniform in [1e14, 2.5e15] FLOP/s, BW log-uniform in
    [1e12, 8e12] B/s, capacities a seeded permutation of {24..288} GiB, link
    bandwidth = BW / 12.5 (the tiny profile's ratio), zero link latency."""
    rng = np.random.Generator(np.random.PCG64(seed))
    caps = np.array([24, 48, 80, 96, 192, 288], dtype=np.float64)
    order = rng.permutation(len(caps))
    out = []
    for h in range(n):
        u, v = rng.random(), rng.random()
        peak = 1.0e14 * 25.0 ** u
        bw = 1.0e12 * 8.0 ** v
        out.append(Hardware(float(peak), float(bw), float(caps[order[h % len(caps)]] * GIB),
                            float(bw / 12.5), 0.0))
    return out


@dataclass(frozen=True)
class Axis:
    """One grid axis: explicit values (u64).  `geom2_start` is set when the values
    are start<<i so that the C ABI can be handed the compact descriptor."""
    values: tuple
    geom2_start: int = 0

    @staticmethod
    def geom2(start: int, count: int) -> "Axis":
        return Axis(tuple(start << i for i in range(count)), start)

    @staticmethod
    def table(vals: Sequence[int]) -> "Axis":
        return Axis(tuple(int(v) for v in vals), 0)

    def __len__(self):
        return len(self.values)

    def array(self) -> np.ndarray:
        return np.asarray(self.values, dtype=np.uint64)


@dataclass(frozen=True)
class Grid:
    """Mixed-radix space; axis order slow -> fast is AXIS_NAMES."""
    models: tuple
    hws: tuple
    axes: tuple  # 9 Axis objects in AXIS_NAMES order (model/hw axes hold table indices)

    @property
    def radices(self):
        return tuple(len(a) for a in self.axes)

    @property
    def size(self) -> int:
        n = 1
        for r in self.radices:
            n *= r
        return n

    def coords(self, idx: int):
        """Digits of a flat index (slowest axis first)."""
        digs = []
        for r in reversed(self.radices):
            digs.append(idx % r)
            idx //= r
        return tuple(reversed(digs))

    def flat(self, digits: Sequence[int]) -> int:
        idx = 0
        for r, dgt in zip(self.radices, digits):
            assert 0 <= dgt < r
            idx = idx * r + dgt
        return idx

    def values_at(self, idx: int):
        return tuple(a.values[dgt] for a, dgt in zip(self.axes, self.coords(idx)))


def make_grid(models, hws, batch, s_in, s_out, tp, wbits, kv_block, mbt) -> Grid:
    return Grid(tuple(models), tuple(hws),
                (Axis.table(range(len(models))), Axis.table(range(len(hws))),
                 batch, s_in, s_out, tp, wbits, kv_block, mbt))


def grid_tiny() -> Grid:
    """1080 rows: 7B-shaped model, one profile, batch 1..256, in 128..4096, out 128..2048, TP 1..8."""
    return make_grid([DENSE_7B], [HW_TINY],
                     Axis.geom2(1, 9), Axis.geom2(128, 6), Axis.geom2(128, 5), Axis.geom2(1, 4),
                     Axis.table([16]), Axis.table([16]), Axis.table([8192]))


def grid_full(seed: int = SEED) -> Grid:
    """1 900 800 rows: 5 models x 6 profiles x 11 x 10 x 8 x 4 x 3 x 2 x 3."""
    return make_grid(MODELS_FULL, hw_profiles(seed),
                     Axis.geom2(1, 11), Axis.geom2(64, 10), Axis.geom2(64, 8), Axis.geom2(1, 4),
                     Axis.table([16, 8, 4]), Axis.table([16, 32]), Axis.table([2048, 4096, 8192]))


def efficiency_pairs(seed: int = SEED, n: int = 64, sigma: float = 0.1):
    """Multiplicative (compute, bandwidth) efficiency factors, each lognormal(0, sigma)."""
    rng = np.random.Generator(np.random.PCG64(seed + 5))
    z = rng.standard_normal((2, n))
    e = np.exp(sigma * z)
    return np.ascontiguousarray(e[0]), np.ascontiguousarray(e[1])


@dataclass(frozen=True)
class Trace:
    """Request trace: unit-rate cumulative arrivals and prompt / generation lengths."""
    arrival_unit: np.ndarray  # f64 [n]
    n_in: np.ndarray          # u32 [n]
    n_out: np.ndarray         # u32 [n]


def request_trace(seed: int = SEED, n: int = N_REQ) -> Trace:
    """Poisson arrivals (unit-rate exponential gaps; divide by the rate per config),
    prompts lognormal(ln 512, 1.0) clipped to [16, 8192], generations
    lognormal(ln 256, 0.8) clipped to [1, 4096]."""
    rng = np.random.Generator(np.random.PCG64(seed + 4))
    gaps = rng.exponential(1.0, n)
    arr = np.cumsum(gaps)
    n_in = np.clip(np.rint(np.exp(np.log(512.0) + 1.0 * rng.standard_normal(n))), 16, 8192)
    n_out = np.clip(np.rint(np.exp(np.log(256.0) + 0.8 * rng.standard_normal(n))), 1, 4096)
    return Trace(np.ascontiguousarray(arr, dtype=np.float64),
                 np.ascontiguousarray(n_in, dtype=np.uint32),
                 np.ascontiguousarray(n_out, dtype=np.uint32))


SIM_RATES = (1.0, 2.0, 4.0, 8.0, 16.0, 32.0, 64.0)


def sim_configs(grid: Grid, n_cfg: int = 65536, seed: int = SEED):
    """Flat indices into `grid` (the batch axis value acts as max concurrent
    sequences; s_in/s_out digits are ignored by the simulator) and an arrival
    rate per simulated config, cycling through SIM_RATES."""
    rng = np.random.Generator(np.random.PCG64(seed + 41))
    idx = rng.integers(0, grid.size, size=n_cfg, dtype=np.uint64).astype(np.uint32)
    rate = np.asarray([SIM_RATES[i % len(SIM_RATES)] for i in range(n_cfg)], dtype=np.float64)
    return np.ascontiguousarray(idx), np.ascontiguousarray(rate)


@dataclass(frozen=True)
class SampleSpace:
    """Tables behind the random-sampled space.  Every per-config draw is a 16-bit
    field of one counter-based random block, mapped to a table index with
    (u16 * n) >> 16, so neither side needs a transcendental function."""
    heads: np.ndarray     # u32[1024]  n_h lattice: round(16 * 8^(j/1023)); hidden = 128*n_h
    peak: np.ndarray      # f64[1024]  1e14 * 25^(j/1023)
    bw: np.ndarray        # f64[1024]  1e12 * 8^(j/1023)
    cap: np.ndarray       # f64[6]
    batch: np.ndarray     # u32[1024]  round(1 * 1024^(j/1023))
    s_in: np.ndarray      # u32[1024]  round(64 * 512^(j/1023))
    s_out: np.ndarray     # u32[1024]  round(64 * 128^(j/1023))
    tp: np.ndarray        # u32[4]
    wbits: np.ndarray     # u32[3]
    kv_block: np.ndarray  # u32[2]
    mbt: np.ndarray       # u32[3]
    kv_choices: np.ndarray = field(default_factory=lambda: np.array([1, 4, 8, 0], dtype=np.uint32))  # 0 = all heads
    layers_lo: int = 16
    layers_n: int = 81        # L uniform in 16..96
    ffn_lo_x2: int = 5        # FFN ratio uniform in [2.5, 4): ratio = (5 + 3*u/65536) / 2
    ffn_span_x2: int = 3
    vocab: int = 32000
    link_div: float = 12.5    # link_bw = bw / 12.5


def sample_space() -> SampleSpace:
    j = np.arange(N_LATTICE, dtype=np.float64) / (N_LATTICE - 1)

    def lat(lo, hi):
        return np.rint(lo * (hi / lo) ** j)

    return SampleSpace(
        heads=lat(16.0, 128.0).astype(np.uint32),
        peak=np.ascontiguousarray(1.0e14 * 25.0 ** j),
        bw=np.ascontiguousarray(1.0e12 * 8.0 ** j),
        cap=np.array([24, 48, 80, 96, 192, 288], dtype=np.float64) * GIB,
        batch=lat(1.0, 1024.0).astype(np.uint32),
        s_in=lat(64.0, 32768.0).astype(np.uint32),
        s_out=lat(64.0, 8192.0).astype(np.uint32),
        tp=np.array([1, 2, 4, 8], dtype=np.uint32),
        wbits=np.array([16, 8, 4], dtype=np.uint32),
        kv_block=np.array([16, 32], dtype=np.uint32),
        mbt=np.array([2048, 4096, 8192], dtype=np.uint32),
    )


# Model-size bucket thresholds of the sampled space: 2^k * 1e9 parameters, k = 0..8.
BUCKET_EDGES = tuple(float(2 ** k) * 1.0e9 for k in range(9))
N_BUCKETS = len(BUCKET_EDGES) + 1
N_HIST_BINS = 256
TTFT_CAP_S = 0.2
SLO_CAPS_S = (0.1, 0.2, 0.5)
