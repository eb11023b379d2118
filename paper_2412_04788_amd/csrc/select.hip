// Selection kernels: constrained per-group top-k by (objective, row) order and
// the two-objective Pareto front.  Reductions run in registers / wave shuffles,
// then LDS per block, then a small second pass over the block partials.
//
// Paper: the simulator evaluates every configuration and keeps the one(s) with
// the least total time (Simulating Hybrid Parallelism); the engine keeps the top
// three by inference time / throughput (Inference Engine, Step 2).
#include "kernels.hpp"
#include "reduce.hpp"

namespace guide {

namespace {

constexpr uint32_t kSelBlocks = 1024;      // upper bound of blocks per reduction pass

struct RowFilter {
    const uint8_t *feasible;
    uint32_t n_con;
    const double *col[GUIDE_MAX_CONSTRAINTS];
    double cap[GUIDE_MAX_CONSTRAINTS];
};

__device__ inline bool row_passes(const RowFilter &f, uint32_t i) {
    bool ok = !f.feasible || f.feasible[i] != 0;
#pragma unroll
    for (uint32_t c = 0; c < GUIDE_MAX_CONSTRAINTS; ++c)
        if (c < f.n_con) ok = ok && (f.col[c][i] <= f.cap[c]);
    return ok;
}

RowFilter make_filter(const guide_select_spec &s) {
    RowFilter f;
    f.feasible = s.feasible;
    f.n_con = s.n_constraints;
    for (uint32_t c = 0; c < GUIDE_MAX_CONSTRAINTS; ++c) {
        f.col[c] = c < s.n_constraints ? s.constraints[c].column : nullptr;
        f.cap[c] = c < s.n_constraints ? s.constraints[c].cap : 0.0;
    }
    return f;
}

uint32_t blocks_for(uint64_t n) {
    uint64_t need = (n + kBlock - 1) / kBlock;
    if (need == 0) need = 1;
    return (uint32_t)(need < kSelBlocks ? need : kSelBlocks);
}

// ------------------------------------------------------------------- top-k

// Workspace layout (u64 units): after_key[G], after_idx[G], part_key[B*G], part_idx[B*G], part_cnt[B*G].
struct TopkWs {
    uint64_t *after_key, *after_idx, *part_key, *part_idx, *part_cnt;
};
TopkWs topk_ws(void *ws, uint32_t G) {
    TopkWs w;
    uint64_t *p = (uint64_t *)ws;
    w.after_key = p; p += GUIDE_MAX_GROUPS;
    w.after_idx = p; p += GUIDE_MAX_GROUPS;
    w.part_key = p; p += (size_t)kSelBlocks * G;
    w.part_idx = p; p += (size_t)kSelBlocks * G;
    w.part_cnt = p;
    return w;
}
size_t topk_ws_bytes(uint32_t G) { return sizeof(uint64_t) * (2 * GUIDE_MAX_GROUPS + 3 * (size_t)kSelBlocks * G); }

// One round: per block and group, the least (key, row) pair strictly after the
// group's previous pick; round 0 also counts passing rows.
// Grouped candidates meet in per-wave LDS slots.  A wave's LDS operations
// execute in program order for all its lanes, so: read the slot, atomic-min the
// key, read back; lanes that hold the new minimum reset the row slot when the
// minimum strictly improved and then atomic-min their row into it.
template <bool GROUPED>
__global__ __launch_bounds__(kBlock) void topk_round_kernel(const double *__restrict__ obj, RowFilter f,
                                                            const uint32_t *__restrict__ group, uint32_t G,
                                                            uint32_t n, uint32_t round, TopkWs w) {
    constexpr int kWaves = kBlock / kWave;
    __shared__ uint64_t s_key[kWaves][GUIDE_MAX_GROUPS], s_idx[kWaves][GUIDE_MAX_GROUPS];
    __shared__ uint32_t s_cnt[kWaves][GUIDE_MAX_GROUPS];
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    for (uint32_t i = threadIdx.x; i < kWaves * GUIDE_MAX_GROUPS; i += kBlock) {
        (&s_key[0][0])[i] = kNone;
        (&s_idx[0][0])[i] = kNone;
        (&s_cnt[0][0])[i] = 0;
    }
    __syncthreads();
    Pair best = {kNone, kNone};
    uint32_t cnt = 0;
    // every lane of a wave runs the same number of iterations (uniform trip count)
    const uint32_t stride = gridDim.x * kBlock;
    const uint32_t iters = (n + stride - 1) / stride;
    for (uint32_t it = 0; it < iters; ++it) {
        const uint32_t i = it * stride + blockIdx.x * kBlock + threadIdx.x;
        bool ok = i < n;
        double x = 0.0;
        uint32_t g = 0;
        if (ok) {
            x = obj[i];
            ok = (x == x) && row_passes(f, i);
            if (GROUPED) {
                g = group[i];
                ok = ok && g < G;
            }
        }
        Pair p = {kNone, kNone};
        if (ok) {
            p.key = key_of(x);
            p.idx = i;
            if (round > 0) {
                const Pair after = {w.after_key[g], w.after_idx[g]};
                ok = less_than(after, p);
            }
        }
        if (!GROUPED) {
            if (ok) best = pair_min(best, p);
            if (round == 0 && p.idx != kNone) ++cnt;
        } else {
            if (round == 0 && p.idx != kNone) atomicAdd(&s_cnt[wave][g], 1u);
            slot_update(s_key[wave], s_idx[wave], g, ok, p);
        }
    }
    if (!GROUPED) {
        best = wave_min(best);
        for (int off = kWave / 2; off > 0; off >>= 1) cnt += __shfl_xor(cnt, off, kWave);
        if (lane == 0) {
            s_key[wave][0] = best.key;
            s_idx[wave][0] = best.idx;
            s_cnt[wave][0] = cnt;
        }
    }
    __syncthreads();
    for (uint32_t g = threadIdx.x; g < G; g += kBlock) {
        Pair b = {s_key[0][g], s_idx[0][g]};
        uint64_t c = s_cnt[0][g];
        for (int wv = 1; wv < kWaves; ++wv) {
            const Pair o = {s_key[wv][g], s_idx[wv][g]};
            b = pair_min(b, o);
            c += s_cnt[wv][g];
        }
        w.part_key[(size_t)blockIdx.x * G + g] = b.key;
        w.part_idx[(size_t)blockIdx.x * G + g] = b.idx;
        if (round == 0) w.part_cnt[(size_t)blockIdx.x * G + g] = c;
    }
}

// One block per group: reduce the block partials, emit pick `round`, remember it.
__global__ __launch_bounds__(kBlock) void topk_final_kernel(TopkWs w, uint32_t G, uint32_t n_blocks, uint32_t round,
                                                            uint32_t k, uint64_t *out_idx, double *out_val,
                                                            uint64_t *out_cnt) {
    __shared__ uint64_t s_key[kBlock / kWave], s_idx[kBlock / kWave], s_cnt[kBlock / kWave];
    const uint32_t g = blockIdx.x;
    Pair best = {kNone, kNone};
    uint64_t cnt = 0;
    for (uint32_t b = threadIdx.x; b < n_blocks; b += kBlock) {
        const Pair o = {w.part_key[(size_t)b * G + g], w.part_idx[(size_t)b * G + g]};
        best = pair_min(best, o);
        if (round == 0) cnt += w.part_cnt[(size_t)b * G + g];
    }
    best = wave_min(best);
    for (int off = kWave / 2; off > 0; off >>= 1) cnt += __shfl_xor(cnt, off, kWave);
    if (threadIdx.x % kWave == 0) {
        s_key[threadIdx.x / kWave] = best.key;
        s_idx[threadIdx.x / kWave] = best.idx;
        s_cnt[threadIdx.x / kWave] = cnt;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int wv = 1; wv < kBlock / kWave; ++wv) {
            const Pair o = {s_key[wv], s_idx[wv]};
            best = pair_min(best, o);
            cnt += s_cnt[wv];
        }
        const bool none = best.idx == kNone;
        out_idx[(size_t)g * k + round] = best.idx;
        out_val[(size_t)g * k + round] = none ? INFINITY : value_of(best.key);
        if (round == 0) out_cnt[g] = cnt;
        // nothing is strictly after (max key, max row): later rounds stay empty
        w.after_key[g] = best.key;
        w.after_idx[g] = best.idx;
    }
}

// --------------------------------------------------------------------- Pareto

constexpr uint32_t kBins = 1u << 16;

// Workspace of the Pareto path.
struct ParetoWs {
    uint64_t *range;      // [2]: min key, max key of x over passing rows
    uint64_t *bin_min;    // [kBins]: least y key per x bin
    uint64_t *bin_lower;  // [kBins]: least y key over strictly lower bins
    uint32_t *bin_cnt;    // [kBins]: survivors per bin
    uint32_t *bin_off;    // [kBins + 1]
    uint32_t *bin_cur;    // [kBins]: scatter cursors
    uint32_t *bin_front;  // [kBins]: front members per bin
    uint32_t *bin_foff;   // [kBins + 1]
    uint32_t *counters;   // [4]: survivors, front size
    uint32_t *surv;       // [n]: surviving rows, arbitrary order
    uint32_t *grouped;    // [n]: surviving rows grouped by bin
    uint8_t *on_front;    // [n]: flag per grouped survivor
};
size_t pareto_ws_bytes(uint64_t n) {
    size_t b = sizeof(uint64_t) * (2 + 2 * (size_t)kBins) + sizeof(uint32_t) * (5 * (size_t)kBins + 2 + 4);
    b += sizeof(uint32_t) * 2 * n + n;
    return b + 256;
}
ParetoWs pareto_ws(void *ws, uint64_t n) {
    ParetoWs w;
    uint64_t *p = (uint64_t *)ws;
    w.range = p; p += 2;
    w.bin_min = p; p += kBins;
    w.bin_lower = p; p += kBins;
    uint32_t *q = (uint32_t *)p;
    w.bin_cnt = q; q += kBins;
    w.bin_off = q; q += kBins + 1;
    w.bin_cur = q; q += kBins;
    w.bin_front = q; q += kBins;
    w.bin_foff = q; q += kBins + 1;
    w.counters = q; q += 4;
    w.surv = q; q += n;
    w.grouped = q; q += n;
    w.on_front = (uint8_t *)q;
    return w;
}

__global__ __launch_bounds__(kBlock) void pareto_init_kernel(ParetoWs w) {
    const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
    if (i < kBins) {
        w.bin_min[i] = kNone;
        w.bin_cnt[i] = 0;
        w.bin_cur[i] = 0;
        w.bin_front[i] = 0;
    }
    if (i == 0) {
        w.range[0] = kNone;
        w.range[1] = 0;
    }
    if (i < 4) w.counters[i] = 0;
}

__device__ inline bool pareto_row(const double *x, const double *y, const RowFilter &f, uint32_t i, uint64_t *kx,
                                  uint64_t *ky) {
    const double xv = x[i], yv = y[i];
    if (!(xv == xv) || !(yv == yv) || !row_passes(f, i)) return false;
    *kx = key_of(xv);
    *ky = key_of(yv);
    return true;
}

__global__ __launch_bounds__(kBlock) void pareto_range_kernel(const double *__restrict__ x, const double *__restrict__ y,
                                                              RowFilter f, uint32_t n, ParetoWs w) {
    uint64_t lo = kNone, hi = 0;
    for (uint32_t i = blockIdx.x * kBlock + threadIdx.x; i < n; i += gridDim.x * kBlock) {
        uint64_t kx, ky;
        if (pareto_row(x, y, f, i, &kx, &ky)) {
            lo = kx < lo ? kx : lo;
            hi = kx > hi ? kx : hi;
        }
    }
    for (int off = kWave / 2; off > 0; off >>= 1) {
        const uint64_t ol = __shfl_xor(lo, off, kWave), oh = __shfl_xor(hi, off, kWave);
        lo = ol < lo ? ol : lo;
        hi = oh > hi ? oh : hi;
    }
    if (threadIdx.x % kWave == 0 && lo != kNone) {
        atomicMin((unsigned long long *)&w.range[0], (unsigned long long)lo);
        atomicMax((unsigned long long *)&w.range[1], (unsigned long long)hi);
    }
}

// Bins are equal slices of the key range of x, so a lower bin means a strictly smaller x.
__device__ inline uint32_t bin_of(uint64_t kx, uint64_t lo, uint32_t shift) { return (uint32_t)((kx - lo) >> shift); }
__device__ inline uint32_t shift_of(uint64_t lo, uint64_t hi) {
    const uint64_t span = hi - lo;
    uint32_t s = 0;
    while (s < 64 && (span >> s) >= kBins) ++s;
    return s;
}

__global__ __launch_bounds__(kBlock) void pareto_binmin_kernel(const double *__restrict__ x, const double *__restrict__ y,
                                                               RowFilter f, uint32_t n, ParetoWs w) {
    const uint64_t lo = w.range[0], hi = w.range[1];
    if (lo == kNone) return;
    const uint32_t shift = shift_of(lo, hi);
    for (uint32_t i = blockIdx.x * kBlock + threadIdx.x; i < n; i += gridDim.x * kBlock) {
        uint64_t kx, ky;
        if (!pareto_row(x, y, f, i, &kx, &ky)) continue;
        const uint32_t b = bin_of(kx, lo, shift);
        // the stored minimum only decreases, so a stale read can only let an extra atomic through
        if (ky < __hip_atomic_load(&w.bin_min[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
            atomicMin((unsigned long long *)&w.bin_min[b], (unsigned long long)ky);
    }
}

// Exclusive prefix (min of bin_min, sum of a count array) over the bins, one block.
__global__ __launch_bounds__(1024) void pareto_scan_min_kernel(ParetoWs w) {
    __shared__ uint64_t s[1024];
    constexpr uint32_t per = kBins / 1024;
    const uint32_t t = threadIdx.x;
    uint64_t m = kNone;
    for (uint32_t j = 0; j < per; ++j) {
        const uint64_t v = w.bin_min[t * per + j];
        m = v < m ? v : m;
    }
    s[t] = m;
    __syncthreads();
    for (uint32_t off = 1; off < 1024; off <<= 1) {
        const uint64_t o = t >= off ? s[t - off] : kNone;
        __syncthreads();
        s[t] = o < s[t] ? o : s[t];
        __syncthreads();
    }
    uint64_t run = t > 0 ? s[t - 1] : kNone;
    for (uint32_t j = 0; j < per; ++j) {
        w.bin_lower[t * per + j] = run;
        const uint64_t v = w.bin_min[t * per + j];
        run = v < run ? v : run;
    }
}

__global__ __launch_bounds__(1024) void scan_sum_kernel(const uint32_t *__restrict__ cnt, uint32_t *__restrict__ off) {
    __shared__ uint32_t s[1024];
    constexpr uint32_t per = kBins / 1024;
    const uint32_t t = threadIdx.x;
    uint32_t m = 0;
    for (uint32_t j = 0; j < per; ++j) m += cnt[t * per + j];
    s[t] = m;
    __syncthreads();
    for (uint32_t o = 1; o < 1024; o <<= 1) {
        const uint32_t v = t >= o ? s[t - o] : 0;
        __syncthreads();
        s[t] += v;
        __syncthreads();
    }
    uint32_t run = t > 0 ? s[t - 1] : 0;
    for (uint32_t j = 0; j < per; ++j) {
        off[t * per + j] = run;
        run += cnt[t * per + j];
    }
    if (t == 1023) off[kBins] = run;
}

// A row survives when its y beats every row of every strictly lower bin; only
// survivors of its own bin can still dominate it.
__global__ __launch_bounds__(kBlock) void pareto_survivors_kernel(const double *__restrict__ x,
                                                                  const double *__restrict__ y, RowFilter f, uint32_t n,
                                                                  ParetoWs w) {
    const uint64_t lo = w.range[0], hi = w.range[1];
    if (lo == kNone) return;
    const uint32_t shift = shift_of(lo, hi);
    const uint32_t stride = gridDim.x * kBlock;
    const uint32_t iters = (n + stride - 1) / stride;
    for (uint32_t it = 0; it < iters; ++it) {
        const uint32_t i = it * stride + blockIdx.x * kBlock + threadIdx.x;
        uint64_t kx, ky;
        bool keep = false;
        uint32_t b = 0;
        if (i < n && pareto_row(x, y, f, i, &kx, &ky)) {
            b = bin_of(kx, lo, shift);
            keep = ky < w.bin_lower[b];
        }
        // wave-aggregated append
        const uint64_t mask = __ballot(keep);
        if (mask) {
            const int lane = threadIdx.x % kWave;
            const int leader = __ffsll((long long)mask) - 1;
            uint32_t base = 0;
            if (lane == leader) base = atomicAdd(&w.counters[0], (uint32_t)__popcll(mask));
            base = __shfl(base, leader, kWave);
            if (keep) {
                w.surv[base + __popcll(mask & ((1ull << lane) - 1))] = i;
                atomicAdd(&w.bin_cnt[b], 1u);
            }
        }
    }
}

__global__ __launch_bounds__(kBlock) void pareto_group_kernel(const double *__restrict__ x, ParetoWs w) {
    const uint32_t m = w.counters[0];
    const uint64_t lo = w.range[0], hi = w.range[1];
    const uint32_t shift = shift_of(lo, hi);
    for (uint32_t s = blockIdx.x * kBlock + threadIdx.x; s < m; s += gridDim.x * kBlock) {
        const uint32_t i = w.surv[s];
        const uint32_t b = bin_of(key_of(x[i]), lo, shift);
        w.grouped[w.bin_off[b] + atomicAdd(&w.bin_cur[b], 1u)] = i;
    }
}

// Exact dominance test against the survivors of the same bin.
__global__ __launch_bounds__(kBlock) void pareto_mark_kernel(const double *__restrict__ x, const double *__restrict__ y,
                                                             ParetoWs w) {
    const uint32_t m = w.counters[0];
    const uint64_t lo = w.range[0], hi = w.range[1];
    const uint32_t shift = shift_of(lo, hi);
    for (uint32_t s = blockIdx.x * kBlock + threadIdx.x; s < m; s += gridDim.x * kBlock) {
        const uint32_t i = w.grouped[s];
        const uint64_t kx = key_of(x[i]), ky = key_of(y[i]);
        const uint32_t b = bin_of(kx, lo, shift);
        bool dominated = false;
        for (uint32_t t = w.bin_off[b]; t < w.bin_off[b + 1] && !dominated; ++t) {
            const uint32_t j = w.grouped[t];
            const uint64_t jx = key_of(x[j]), jy = key_of(y[j]);
            dominated = jx <= kx && jy <= ky && (jx < kx || jy < ky);
        }
        w.on_front[s] = dominated ? 0 : 1;
        if (!dominated) atomicAdd(&w.bin_front[b], 1u);
    }
}

// Position of a front member = front members of lower bins + members of its own
// bin that precede it in (x, y, row) order.
__global__ __launch_bounds__(kBlock) void pareto_emit_kernel(const double *__restrict__ x, const double *__restrict__ y,
                                                             ParetoWs w, uint64_t *out_idx, uint64_t capacity,
                                                             uint64_t *out_count) {
    const uint32_t m = w.counters[0];
    const uint64_t lo = w.range[0], hi = w.range[1];
    const uint32_t shift = shift_of(lo, hi);
    if (blockIdx.x == 0 && threadIdx.x == 0) out_count[0] = lo == kNone ? 0 : w.bin_foff[kBins];
    for (uint32_t s = blockIdx.x * kBlock + threadIdx.x; s < m; s += gridDim.x * kBlock) {
        if (!w.on_front[s]) continue;
        const uint32_t i = w.grouped[s];
        const uint64_t kx = key_of(x[i]), ky = key_of(y[i]);
        const uint32_t b = bin_of(kx, lo, shift);
        uint32_t rank = 0;
        for (uint32_t t = w.bin_off[b]; t < w.bin_off[b + 1]; ++t) {
            if (!w.on_front[t]) continue;
            const uint32_t j = w.grouped[t];
            const uint64_t jx = key_of(x[j]), jy = key_of(y[j]);
            if (jx < kx || (jx == kx && (jy < ky || (jy == ky && j < i)))) ++rank;
        }
        const uint64_t pos = (uint64_t)w.bin_foff[b] + rank;
        if (pos < capacity) out_idx[pos] = i;
    }
}

__global__ void pareto_empty_kernel(uint64_t *out_count) { out_count[0] = 0; }

}  // namespace

size_t select_workspace_bytes(const guide_select_spec &spec, uint64_t n) {
    if (spec.mode == GUIDE_SELECT_PARETO) return pareto_ws_bytes(n);
    return topk_ws_bytes(spec.n_groups ? spec.n_groups : 1);
}

hipError_t launch_select_topk(const guide_select_spec &spec, uint64_t n, const guide_select_out &out, void *ws,
                              hipStream_t stream) {
    const uint32_t G = spec.n_groups;
    const TopkWs w = topk_ws(ws, G);
    const RowFilter f = make_filter(spec);
    const uint32_t nb = blocks_for(n);
    for (uint32_t round = 0; round < spec.k; ++round) {
        if (spec.group)
            hipLaunchKernelGGL(topk_round_kernel<true>, dim3(nb), dim3(kBlock), 0, stream, spec.objective, f, spec.group,
                               G, (uint32_t)n, round, w);
        else
            hipLaunchKernelGGL(topk_round_kernel<false>, dim3(nb), dim3(kBlock), 0, stream, spec.objective, f,
                               (const uint32_t *)nullptr, G, (uint32_t)n, round, w);
        hipLaunchKernelGGL(topk_final_kernel, dim3(G), dim3(kBlock), 0, stream, w, G, nb, round, spec.k, out.idx, out.val,
                           out.count);
    }
    return hipGetLastError();
}

hipError_t launch_select_pareto(const guide_select_spec &spec, uint64_t n, const guide_select_out &out, void *ws,
                                hipStream_t stream) {
    if (n == 0) {
        hipLaunchKernelGGL(pareto_empty_kernel, dim3(1), dim3(1), 0, stream, out.count);
        return hipGetLastError();
    }
    const ParetoWs w = pareto_ws(ws, n);
    const RowFilter f = make_filter(spec);
    const uint32_t nb = blocks_for(n), n32 = (uint32_t)n;
    const double *x = spec.objective, *y = spec.objective_y;
    hipLaunchKernelGGL(pareto_init_kernel, dim3(kBins / kBlock), dim3(kBlock), 0, stream, w);
    hipLaunchKernelGGL(pareto_range_kernel, dim3(nb), dim3(kBlock), 0, stream, x, y, f, n32, w);
    hipLaunchKernelGGL(pareto_binmin_kernel, dim3(nb), dim3(kBlock), 0, stream, x, y, f, n32, w);
    hipLaunchKernelGGL(pareto_scan_min_kernel, dim3(1), dim3(1024), 0, stream, w);
    hipLaunchKernelGGL(pareto_survivors_kernel, dim3(nb), dim3(kBlock), 0, stream, x, y, f, n32, w);
    hipLaunchKernelGGL(scan_sum_kernel, dim3(1), dim3(1024), 0, stream, (const uint32_t *)w.bin_cnt, w.bin_off);
    hipLaunchKernelGGL(pareto_group_kernel, dim3(nb), dim3(kBlock), 0, stream, x, w);
    hipLaunchKernelGGL(pareto_mark_kernel, dim3(nb), dim3(kBlock), 0, stream, x, y, w);
    hipLaunchKernelGGL(scan_sum_kernel, dim3(1), dim3(1024), 0, stream, (const uint32_t *)w.bin_front, w.bin_foff);
    hipLaunchKernelGGL(pareto_emit_kernel, dim3(nb), dim3(kBlock), 0, stream, x, y, w, out.idx, out.capacity, out.count);
    return hipGetLastError();
}

}  // namespace guide
