// Grid evaluation kernels: flat index -> mixed-radix digits -> candidate ->
// metrics, one candidate per lane, spec tables staged in LDS, coalesced
// structure-of-arrays stores.
#include <hip/hip_ext.h>

#include "kernels.hpp"
#include "perf_model.hpp"
#include "select_shared.hpp"

namespace guide {

struct GridLds {
    uint32_t axis[kNumAxes][GUIDE_MAX_AXIS_VALUES];
    guide_model models[GUIDE_MAX_MODELS];
    HwRecip hw[GUIDE_MAX_HW];
};

__device__ inline void stage_grid_tables(GridLds &s, const GridDesc &g, const DevTables *__restrict__ tab) {
    for (uint32_t i = threadIdx.x; i < kNumAxes * GUIDE_MAX_AXIS_VALUES; i += blockDim.x)
        (&s.axis[0][0])[i] = (&tab->axis_vals[0][0])[i];
    for (uint32_t i = threadIdx.x; i < g.n_models * 8u; i += blockDim.x)
        ((uint32_t *)s.models)[i] = ((const uint32_t *)tab->models)[i];
    for (uint32_t i = threadIdx.x; i < g.n_hw; i += blockDim.x) {
        const guide_hw h = tab->hw[i];
        HwRecip r;
        r.r_peak = 1.0 / h.peak_flops;
        r.r_bw = 1.0 / h.hbm_bw;
        r.cap = h.cap_bytes;
        r.r_link = 1.0 / h.link_bw;
        r.lat = h.link_lat;
        s.hw[i] = r;
    }
}

struct Candidate {
    uint32_t model, hw;
    Knobs kn;
};

__device__ inline Candidate decode_index(const GridLds &s, const GridDesc &g, uint32_t idx) {
    uint32_t v[kNumAxes];
    uint32_t rem = idx;
#pragma unroll
    for (int a = kNumAxes - 1; a > 0; --a) {
        const uint32_t q = div32(rem, g.div[a]);
        v[a] = s.axis[a][rem - q * g.div[a].d];
        rem = q;
    }
    v[0] = s.axis[0][rem];
    Candidate c;
    c.model = v[AX_MODEL];
    c.hw = v[AX_HW];
    c.kn.b = v[AX_BATCH];
    c.kn.s_in = v[AX_SIN];
    c.kn.s_out = v[AX_SOUT];
    c.kn.p = v[AX_TP];
    c.kn.wbits = v[AX_WBITS];
    c.kn.blk = v[AX_BLK];
    c.kn.mbt = v[AX_MBT];
    return c;
}

// GPU-hours per million generated tokens.
__device__ inline double cost_of(const Knobs &kn, double t_batch) {
    return (double)kn.p * t_batch / 3600.0 * 1.0e6 / ((double)kn.b * (double)kn.s_out);
}

template <bool ADDITIVE>
__global__ __launch_bounds__(kBlock) void eval_grid_kernel(GridDesc g, const DevTables *__restrict__ tab,
                                                           uint32_t first, uint32_t count, double re_c, double re_b,
                                                           guide_metrics out) {
    __shared__ GridLds s;
    stage_grid_tables(s, g, tab);
    __syncthreads();
    for (uint32_t i = blockIdx.x * kBlock + threadIdx.x; i < count; i += gridDim.x * kBlock) {
        const Candidate c = decode_index(s, g, first + i);
        const Coef cf = make_coef(s.models[c.model], c.kn.p, c.kn.wbits);
        const HwRecip hw = s.hw[c.hw];
        const TimeCoef tc = make_time_coef(cf, hw.r_peak * re_c, hw.r_bw * re_b, hw.r_link, hw.lat);
        const EvalResult r = evaluate_times<ADDITIVE>(tc, c.kn);
        const MemResult m = memory_check(cf, hw.cap, c.kn.b, c.kn.s_in, c.kn.s_out, c.kn.blk);
        const double t_batch = r.t_prefill + r.t_decode;
        if (out.t_prefill) out.t_prefill[i] = r.t_prefill;
        if (out.t_decode) out.t_decode[i] = r.t_decode;
        if (out.t_batch) out.t_batch[i] = t_batch;
        if (out.decode_tok_s) {
            const double n = (double)(c.kn.s_out - 1);
            out.decode_tok_s[i] = c.kn.s_out > 1 ? (double)c.kn.b * n / r.t_decode : 0.0;
        }
        if (out.cost) out.cost[i] = cost_of(c.kn, t_batch);
        if (out.b_max) out.b_max[i] = m.b_max;
        if (out.feasible) out.feasible[i] = m.feasible ? 1 : 0;
    }
}

// ---------------------------------------------------------------- tiled variant
//
// The two fastest axes (KV block, max batched tokens) change only part of the
// model: the decode series does not depend on either, the prefill only on the
// token budget, the memory check only on the block size.  A lane therefore takes
// one *tile* = all NB x NM combinations of those two axes for one setting of the
// seven slower axes (NB*NM consecutive flat indices), evaluates the shared parts
// once, and the wave transposes each output column through LDS so that global
// stores stay coalesced (lane l stores index base + 64*it + l).

// What a block needs besides the index range is the same for every block and every call on an
// unchanged grid: the axis values, models and hardware reciprocals, the nudged reciprocals of the
// divisors, and the per-op FLOPs / bytes of every (model, tp, precision) combination.  A one-block
// kernel derives them once into device memory (when the context's tables change); the evaluation
// blocks copy them into LDS.
constexpr uint32_t kCoefRows = 96;          // (model, tp, precision) rows of per-op coefficients kept in LDS
struct alignas(16) TileLds {
    GridLds g;
    double r_tp[GUIDE_MAX_AXIS_VALUES];     // 1 / tp
    double r_sin[GUIDE_MAX_AXIS_VALUES];    // nudged reciprocals for exact floor division
    double r_blk[GUIDE_MAX_AXIS_VALUES];
    double r_mbt[GUIDE_MAX_AXIS_VALUES];
    Coef coef[kCoefRows];                   // last: only the rows in use are copied
};
static_assert(offsetof(TileLds, coef) % 16 == 0 && sizeof(TileLds) % 16 == 0, "copied in 16-byte words");

__global__ __launch_bounds__(kBlock) void tile_tables_kernel(GridDesc g, const DevTables *__restrict__ tab,
                                                             TileLds *__restrict__ dst) {
    stage_grid_tables(dst->g, g, tab);
    for (uint32_t i = threadIdx.x; i < GUIDE_MAX_AXIS_VALUES; i += blockDim.x) {
        dst->r_tp[i] = 1.0 / (double)max(tab->axis_vals[AX_TP][i], 1u);
        dst->r_sin[i] = recip_up(1.0 / (double)max(tab->axis_vals[AX_SIN][i], 1u));
        dst->r_blk[i] = recip_up(1.0 / (double)max(tab->axis_vals[AX_BLK][i], 1u));
        dst->r_mbt[i] = recip_up(1.0 / (double)max(tab->axis_vals[AX_MBT][i], 1u));
    }
    const uint32_t n_tp = g.div[AX_TP].d, n_w = g.div[AX_WBITS].d;
    const uint32_t n_rows = g.div[AX_MODEL].d * n_tp * n_w;
    if (n_rows <= kCoefRows) {
        for (uint32_t r = threadIdx.x; r < n_rows; r += blockDim.x) {
            const uint32_t dw = r % n_w, dt = (r / n_w) % n_tp, dm = r / (n_w * n_tp);
            const uint32_t p = tab->axis_vals[AX_TP][dt];
            dst->coef[r] = make_coef(tab->models[tab->axis_vals[AX_MODEL][dm]], p, tab->axis_vals[AX_WBITS][dw],
                                     1.0 / (double)p);
        }
    }
}

// Row sample for a Pareto selection over the rows being evaluated, taken by extra blocks of the evaluation kernel
// (block `rb` of them; kBlock samples each): sample_number / sample_row give the rows.  The
// sampled rows are evaluated here from scratch rather than read back, so the sample does not wait for the columns.
// It fixes the range of x that the selection's bins slice (any range is correct, a good one is fast), and the
// block hands the front of its sample rows to the selection's filter pass (store_sample_front).
// Also resets the counters that the selection's kernels accumulate into.
constexpr uint64_t kSampleMargin = 1ull << 26;      // in key units: 2^-26 relative for a normal number
template <bool ADDITIVE>
__device__ inline void sample_rider(const GridLds &s, const GridDesc &g, uint32_t rb, uint32_t n_rider_blocks, uint32_t first,
                                    uint32_t count, double re_c, double re_b, const FusedSelect &fs) {
    constexpr int kWaves = kBlock / kWave;
    __shared__ uint64_t s_lo[kWaves];
    __shared__ Pair s_best[kWaves];
    SelectScratch *sc = (SelectScratch *)fs.scratch;
    const uint32_t gid = rb * kBlock + threadIdx.x;
    const uint32_t n_samples = n_rider_blocks * kBlock;
    if (gid == 0) sc->counters[0] = sc->counters[1] = 0;
    const uint32_t stride = count > n_samples ? count / n_samples : 1;
    const uint32_t k = sample_number(rb, n_rider_blocks);
    uint64_t lo = kNone, kx = 0, ky = 0;
    Pair best = {kNone, kNone};
    bool pass = false;
    if ((uint64_t)k * stride < count) {
        const Candidate c = decode_index(s, g, first + sample_row(k, stride));
        const Coef cf = make_coef(s.models[c.model], c.kn.p, c.kn.wbits);
        const HwRecip hw = s.hw[c.hw];
        const TimeCoef tc = make_time_coef(cf, hw.r_peak * re_c, hw.r_bw * re_b, hw.r_link, hw.lat);
        const EvalResult r = evaluate_times<ADDITIVE>(tc, c.kn);
        const double t_batch = r.t_prefill + r.t_decode;
        const double tok_s = c.kn.s_out > 1 ? (double)c.kn.b * (double)(c.kn.s_out - 1) / r.t_decode : 0.0;
        const double cost = cost_of(c.kn, t_batch);
        auto col = [&](uint32_t id) {
            return id == GUIDE_COL_T_PREFILL ? r.t_prefill
                   : id == GUIDE_COL_T_DECODE ? r.t_decode
                   : id == GUIDE_COL_T_BATCH ? t_batch
                   : id == GUIDE_COL_DECODE_TOK_S ? tok_s : cost;
        };
        // The values here come from another instruction sequence than the stored columns and may differ
        // from them in the last bits (every sequence is within 1e-9 relative of the definition), while a
        // sample row may only prune rows that the stored row dominates.  So the sample row is moved up by
        // 2^-26 relative in x and y (a point that the stored row dominates prunes no row wrongly), and it
        // must pass its filter by the same margin (a row that is not a passing row must prune nothing).
        const double x = col(fs.pareto_x), y = col(fs.pareto_y);
        bool ok = x == x && y == y;
        for (uint32_t q = 0; q < fs.pareto_filter.n_con; ++q) {
            const double v = col(fs.pareto_filter.col[q]), cap = fs.pareto_filter.cap[q];
            ok = ok && v == v && cap == cap && key_of(v) + kSampleMargin <= key_of(cap);
        }
        if (ok && fs.pareto_filter.use_feasible) {
            const double c_avail = hw.cap - cf.w_gpu;
            const uint32_t tok_req = (c.kn.s_in + c.kn.s_out + c.kn.blk - 1) / c.kn.blk * c.kn.blk;
            ok = c_avail > 0.0 && (double)c.kn.b * ((double)tok_req * cf.kv_tok) * (1.0 + 0x1p-26) <= c_avail;
        }
        if (ok) {
            pass = true;
            lo = kx = key_of(x);
            ky = key_of(y);
            best = Pair{ky, kx};
        }
    }
    lo = wave_min(lo);
    best = wave_min(best);
    if (threadIdx.x % kWave == 0) {
        s_lo[threadIdx.x / kWave] = lo;
        s_best[threadIdx.x / kWave] = best;
    }
    store_sample_front(pass, kx + kSampleMargin, ky + kSampleMargin, sc->sample_front + rb * kSampleFrontPer);
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int wv = 1; wv < kWaves; ++wv) {
            lo = min_u64(lo, s_lo[wv]);
            best = pair_min(best, s_best[wv]);
        }
        sc->sample_lo[rb] = lo;
        sc->sample_best[rb] = best;
    }
}

// FUSED: a top-k folded in (FusedSelect); every block then writes its top-K partials, also when it owns no tile.
// STREAM: full waves store the 8-byte columns with the streaming hint.
template <bool ADDITIVE, int NB, int NM, bool FUSED, bool STREAM>
__global__ __launch_bounds__(kBlock) void eval_tile_kernel(GridDesc g, const DevTables *__restrict__ tab,
                                                           uint32_t first, uint32_t count, double re_c, double re_b,
                                                           guide_metrics out, FusedSelect fs,
                                                           const TileLds *__restrict__ derived) {
    constexpr int TS = NB * NM;
    constexpr int kWaves = kBlock / kWave;
    __shared__ TileLds s;
    __shared__ double s_x[kWaves][kWave * TS];
    const uint32_t n_tp = g.div[AX_TP].d, n_w = g.div[AX_WBITS].d;
    const uint32_t n_rows = g.div[AX_MODEL].d * n_tp * n_w;
    const bool coef_in_lds = n_rows <= kCoefRows;
    {
        // every load is issued before the first LDS write, so the copy costs one memory latency
        const uint32_t vecs = (uint32_t)(offsetof(TileLds, coef) + (coef_in_lds ? n_rows : 0u) * sizeof(Coef) + 15) / 16;
        constexpr uint32_t kPer = (sizeof(TileLds) / 16 + kBlock - 1) / kBlock;
        const uint4 *src = (const uint4 *)derived;
        uint4 *dst = (uint4 *)&s;
        uint4 t[kPer];
#pragma unroll
        for (uint32_t q = 0; q < kPer; ++q) {
            const uint32_t i = q * kBlock + threadIdx.x;
            t[q] = i < vecs ? src[i] : uint4{0, 0, 0, 0};
        }
#pragma unroll
        for (uint32_t q = 0; q < kPer; ++q) {
            const uint32_t i = q * kBlock + threadIdx.x;
            if (i < vecs) dst[i] = t[q];
        }
    }
    TopList<kFusedTopK> top;
    uint64_t n_pass = 0, top_bound = kNone;
    uint32_t batch = 0;
    if (FUSED) top.init();
    __syncthreads();
    if (fs.rider_blocks && blockIdx.x >= gridDim.x - fs.rider_blocks) {                // block-uniform
        sample_rider<ADDITIVE>(s.g, g, blockIdx.x - (gridDim.x - fs.rider_blocks), fs.rider_blocks, first, count, re_c,
                               re_b, fs);
        return;
    }
    const uint32_t n_main_blocks = gridDim.x - fs.rider_blocks;
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    double *xw = s_x[wave];
    const uint32_t t_first = first / TS;
    const uint32_t n_tiles = (first + count - 1) / TS - t_first + 1;
    const uint32_t last = first + count;                       // exclusive; count > 0, no overflow (grid < 2^32)
    for (uint32_t tb = (blockIdx.x * kWaves + wave) * kWave; tb < n_tiles; tb += n_main_blocks * kWaves * kWave) {
        const uint32_t tl = tb + lane < n_tiles ? tb + lane : n_tiles - 1;   // idle lanes repeat the last tile
        // digits of the seven slow axes
        uint32_t dg[AX_BLK];
        uint32_t rem = t_first + tl;
#pragma unroll
        for (int a = AX_BLK - 1; a > 0; --a) {
            const uint32_t q = div32(rem, g.div[a]);
            dg[a] = rem - q * g.div[a].d;
            rem = q;
        }
        dg[0] = rem;
        Knobs kn;
        kn.b = s.g.axis[AX_BATCH][dg[AX_BATCH]];
        kn.s_in = s.g.axis[AX_SIN][dg[AX_SIN]];
        kn.s_out = s.g.axis[AX_SOUT][dg[AX_SOUT]];
        kn.p = s.g.axis[AX_TP][dg[AX_TP]];
        kn.wbits = s.g.axis[AX_WBITS][dg[AX_WBITS]];
        const Coef cf = coef_in_lds
                            ? s.coef[(dg[AX_MODEL] * n_tp + dg[AX_TP]) * n_w + dg[AX_WBITS]]
                            : make_coef(s.g.models[s.g.axis[AX_MODEL][dg[AX_MODEL]]], kn.p, kn.wbits, s.r_tp[dg[AX_TP]]);
        const HwRecip hw = s.g.hw[s.g.axis[AX_HW][dg[AX_HW]]];
        const TimeCoef tc = make_time_coef(cf, hw.r_peak * re_c, hw.r_bw * re_b, hw.r_link, hw.lat);

        // coalesced stores: element e of the wave's 64*TS consecutive indices sits in lane e / TS, slot e % TS.
        // Columns leave as soon as their values exist so that stores overlap the remaining arithmetic.
        const uint32_t cfg0 = (t_first + tb) * TS;             // flat index of the wave's first element
        // every element of the wave inside [first, last): no per-element checks (wave-uniform)
        const bool full = tb + kWave <= n_tiles && cfg0 >= first && cfg0 + kWave * TS <= last;
        auto store_f64 = [&](double *col, auto value_of_slot) {
            if (!col) return;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
            for (int j = 0; j < TS; ++j) xw[lane * TS + j] = value_of_slot(j);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            if (full) {
                double *dst = col + (cfg0 - first) + lane;
#pragma unroll
                for (int it = 0; it < TS; ++it) {
                    if (STREAM) __builtin_nontemporal_store(xw[it * kWave + lane], &dst[it * kWave]);
                    else dst[it * kWave] = xw[it * kWave + lane];
                }
            } else {
#pragma unroll
                for (int it = 0; it < TS; ++it) {
                    const uint32_t cfg = cfg0 + it * kWave + lane;
                    const double v = xw[it * kWave + lane];
                    if (cfg >= first && cfg < last && tb + (it * kWave + lane) / TS < n_tiles) col[cfg - first] = v;
                }
            }
        };

        // memory check: depends on the block size only
        MemResult mem[NB];
        const bool need_mem = out.b_max || out.feasible ||
                              (FUSED && fs.topk && fs.topk_filter.use_feasible);
        if (need_mem) {
            const double c_avail = hw.cap - cf.w_gpu;
            const uint32_t tok = kn.s_in + kn.s_out;
#pragma unroll
            for (int k = 0; k < NB; ++k) {
                const uint32_t blk = s.g.axis[AX_BLK][k];
                const uint32_t tok_req = floor_div(tok + blk - 1, s.r_blk[k]) * blk;
                const double kv_req = (double)tok_req * cf.kv_tok;
                const double q = floor(c_avail / kv_req);
                const bool room = c_avail > 0.0;
                mem[k].feasible = room && (double)kn.b * kv_req <= c_avail;
                mem[k].b_max = !room ? 0u : (q >= 4294967295.0 ? 4294967295u : (uint32_t)q);
            }
        }
        if (out.b_max || out.feasible) {
            uint32_t *xi = (uint32_t *)xw;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
            for (int j = 0; j < TS; ++j) {
                xi[lane * TS + j] = mem[j / NM].b_max;
                xi[kWave * TS + lane * TS + j] = mem[j / NM].feasible ? 1u : 0u;
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
            for (int it = 0; it < TS; ++it) {
                const uint32_t cfg = cfg0 + it * kWave + lane;
                const uint32_t bm = xi[it * kWave + lane], fe = xi[kWave * TS + it * kWave + lane];
                if (full || (cfg >= first && cfg < last && tb + (it * kWave + lane) / TS < n_tiles)) {
                    if (out.b_max) out.b_max[cfg - first] = bm;
                    if (out.feasible) out.feasible[cfg - first] = (uint8_t)fe;
                }
            }
        }

        // decode series: depends on neither tile axis
        const double t_decode = decode_time_fast<ADDITIVE>(tc, kn.b, kn.s_in, kn.s_out - 1);
        const double tok_s = kn.s_out > 1 ? (double)kn.b * (double)(kn.s_out - 1) * fast_recip(t_decode) : 0.0;
        store_f64(out.t_decode, [&](int) { return t_decode; });
        store_f64(out.decode_tok_s, [&](int) { return tok_s; });

        // prefill: depends on the token budget only
        double t_prefill[NM];
#pragma unroll
        for (int m = 0; m < NM; ++m)
            t_prefill[m] = prefill_time_fast<ADDITIVE>(tc, kn.b, kn.s_in, s.g.axis[AX_MBT][m], s.r_sin[dg[AX_SIN]],
                                                        s.r_mbt[m]);
        const double bs = (double)kn.b * (double)kn.s_out;
        const double cost_f = (double)kn.p * (1.0e6 / 3600.0) * fast_recip(bs);
        double t_batch[NM], cost[NM];
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            t_batch[m] = t_prefill[m] + t_decode;
            cost[m] = t_batch[m] * cost_f;
        }
        store_f64(out.t_prefill, [&](int j) { return t_prefill[j % NM]; });
        store_f64(out.t_batch, [&](int j) { return t_batch[j % NM]; });
        store_f64(out.cost, [&](int j) { return cost[j % NM]; });

        if (FUSED) {
            // The selections see exactly the values stored above.  A column's value depends on the
            // token-budget digit m at most and feasibility on the block-size digit k only, so the
            // filters and keys are worked out once per m and each row costs a few compares.
            const bool tile_real = tb + lane < n_tiles;
            const uint32_t row0 = (t_first + tl) * TS;
            auto col = [&](uint32_t id, int m) {
                return id == GUIDE_COL_T_PREFILL ? t_prefill[m]
                       : id == GUIDE_COL_T_DECODE ? t_decode
                       : id == GUIDE_COL_T_BATCH ? t_batch[m]
                       : id == GUIDE_COL_DECODE_TOK_S ? tok_s : cost[m];
            };
            auto passes = [&](const FusedFilter &f, int m) {
                bool ok = true;
                for (uint32_t c = 0; c < f.n_con; ++c) ok = ok && (col(f.col[c], m) <= f.cap[c]);
                return ok;
            };
            if (fs.topk) {
                uint64_t key[NM];
                bool ok_m[NM], cand = false;
                uint32_t n_ok = 0;
#pragma unroll
                for (int m = 0; m < NM; ++m) {
                    const double v = col(fs.topk_obj, m);
                    key[m] = key_of(v);
                    ok_m[m] = tile_real && v == v && passes(fs.topk_filter, m);
                    n_ok += ok_m[m] ? 1u : 0u;
                    cand = cand || (ok_m[m] && key[m] <= top_bound);
                }
                auto feas = [&](int k) { return !fs.topk_filter.use_feasible || mem[k].feasible; };
                if (full) {
                    // every row of the wave's tiles is in range: passing rows are counted per tile, and the
                    // rows are visited only when one of them can still enter the list
                    uint32_t n_f = 0;
#pragma unroll
                    for (int k = 0; k < NB; ++k) n_f += feas(k) ? 1u : 0u;
                    n_pass += n_ok * n_f;
                    if (cand) {
#pragma unroll
                        for (int j = 0; j < TS; ++j) {
                            const int k = j / NM, m = j % NM;
                            if (ok_m[m] && feas(k) && key[m] <= top_bound)
                                top.insert_ascending(Pair{key[m], (uint64_t)(row0 + j - first)});
                        }
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < TS; ++j) {
                        const int k = j / NM, m = j % NM;
                        const uint32_t row = row0 + j;
                        if (ok_m[m] && row >= first && row < last && feas(k)) {
                            ++n_pass;
                            if (key[m] <= top_bound) top.insert_ascending(Pair{key[m], (uint64_t)(row - first)});
                        }
                    }
                }
                // Some lane already holds K keys at or below the least K-th key of the wave's lanes, so a
                // row above it cannot be among the block's K least.  The bound tightens fast at first and
                // slowly later: refreshed after each of the first four batches, then after every fourth.
                if (batch < 4 || (batch & 3) == 0) top_bound = wave_min(top.v[kFusedTopK - 1].key);
                ++batch;
            }
        }
    }
    if (FUSED) {
        constexpr int kCap = 8;
        __shared__ Pair s_pairs[kWaves][kFusedTopK], s_cand[kWaves][kCap];
        __shared__ uint32_t s_n[kWaves];
        __shared__ uint64_t s_cnt[kWaves];
        if (fs.topk) {
            const Top1Ws w = top1_ws(fs.topk_ws);
            for (int off = kWave / 2; off > 0; off >>= 1) n_pass += __shfl_xor(n_pass, off, kWave);
            if (lane == 0) s_cnt[wave] = n_pass;
            top_bound = wave_min(top.v[kFusedTopK - 1].key);
            block_topk_bounded<kFusedTopK, kWaves, kCap>(top, top_bound, s_cand, s_n, s_pairs, [&](int r, const Pair &p) {
                w.key[(size_t)blockIdx.x * kFusedTopK + r] = p.key;
                w.idx[(size_t)blockIdx.x * kFusedTopK + r] = p.idx;
            });                                          // (contains the barrier that publishes s_cnt)
            if (threadIdx.x == 0) {
                uint64_t c = 0;
                for (int wv = 0; wv < kWaves; ++wv) c += s_cnt[wv];
                w.cnt[blockIdx.x] = c;
            }
        }
    }
}

// The R smallest (LARGEST: largest) values seen, kept sorted with the extreme one first; R <= 7 covers the
// nearest-rank p10 / p90 of up to 64 samples.  Values arrive eight at a time, already sorted ascending
// (merge), or one by one (push).  Compare-exchanges are a minimum and a maximum.
constexpr int kRankMax = 7;
constexpr int kSweepGroup = 8;
template <bool LARGEST>
struct ExtremeK {
    double v[kRankMax];
    // puts the value that belongs nearer the front of the list into a
    static __device__ void cx(double &a, double &b) {
        const double lo = fmin(a, b), hi = fmax(a, b);
        a = LARGEST ? hi : lo;
        b = LARGEST ? lo : hi;
    }
    __device__ void init() {
#pragma unroll
        for (int i = 0; i < kRankMax; ++i) v[i] = LARGEST ? -INFINITY : INFINITY;
    }
    __device__ void push(double x) {
#pragma unroll
        for (int i = 0; i < kRankMax; ++i) cx(v[i], x);
    }
    // a[0] <= ... <= a[7].  Entry i of the list meets the i-th candidate from the other end of the group's seven
    // best (the eighth cannot be among the seven best of the union): the better of each pair are the union's
    // seven best, in a sequence that rises and falls once, which the last three stages of a bitonic sorter of
    // eight put in order (its first element would be a sentinel that no exchange moves, so those are left out).
    __device__ void merge(const double (&a)[kSweepGroup]) {
        double w[kSweepGroup];
#pragma unroll
        for (int i = 0; i < kRankMax; ++i) {
            const double c = LARGEST ? a[1 + i] : a[kRankMax - 1 - i];
            w[1 + i] = LARGEST ? fmax(v[i], c) : fmin(v[i], c);
        }
        cx(w[1], w[5]); cx(w[2], w[6]); cx(w[3], w[7]);
        cx(w[1], w[3]); cx(w[4], w[6]); cx(w[5], w[7]);
        cx(w[2], w[3]); cx(w[4], w[5]); cx(w[6], w[7]);
#pragma unroll
        for (int i = 0; i < kRankMax; ++i) v[i] = w[1 + i];
    }
    __device__ double at(uint32_t r) const {   // r-th from the extreme end, 0-based
        double x = v[0];
#pragma unroll
        for (int i = 1; i < kRankMax; ++i) x = r == (uint32_t)i ? v[i] : x;
        return x;
    }
};
// Eight values in ascending order (19 compare-exchanges).
__device__ inline void sort_group(double (&a)[kSweepGroup]) {
    auto cx = [](double &x, double &y) {
        const double lo = fmin(x, y), hi = fmax(x, y);
        x = lo;
        y = hi;
    };
    cx(a[0], a[1]); cx(a[2], a[3]); cx(a[4], a[5]); cx(a[6], a[7]);
    cx(a[0], a[2]); cx(a[1], a[3]); cx(a[4], a[6]); cx(a[5], a[7]);
    cx(a[1], a[2]); cx(a[5], a[6]); cx(a[0], a[4]); cx(a[3], a[7]);
    cx(a[1], a[5]); cx(a[2], a[6]);
    cx(a[1], a[4]); cx(a[3], a[6]);
    cx(a[2], a[4]); cx(a[3], a[5]);
    cx(a[3], a[4]);
}

// Efficiency sweep.  Neither latency depends on the KV block size, so one lane evaluates the samples
// for all block sizes of a configuration at once (rows that differ only in the kv_block digit) and
// only the memory check is repeated per block size; the split of the prefill into passes does not
// depend on the sample and is planned once.
// Two waves per SIMD: the register budget that asks for costs a few spills, and measured 0.44 ms against 0.56 ms
// with one wave (three and four waves spill far more: 1.5 and 2.7 ms).
template <bool ADDITIVE>
__global__ __launch_bounds__(kBlock, 2) void eval_sweep_kernel(GridDesc g, const DevTables *__restrict__ tab,
                                                            uint32_t first, uint32_t count, uint32_t n_eff,
                                                            guide_stats out) {
    __shared__ GridLds s;
    __shared__ double s_rec[GUIDE_MAX_EFF], s_reb[GUIDE_MAX_EFF];
    stage_grid_tables(s, g, tab);
    for (uint32_t i = threadIdx.x; i < n_eff; i += blockDim.x) {
        s_rec[i] = 1.0 / tab->eff_c[i];
        s_reb[i] = 1.0 / tab->eff_b[i];
    }
    __syncthreads();
    // nearest rank: p10 = sorted[ceil(n/10) - 1]; p90 = sorted[ceil(9n/10) - 1] = (n - ceil(9n/10))-th largest, 0-based
    const uint32_t r_lo = (n_eff + 9) / 10 - 1;
    const uint32_t r_hi = n_eff - (9 * n_eff + 9) / 10;
    // work item u = (index with the kv_block digit removed): rows (hi * NB + k) * NM + m for k < NB
    const uint32_t NB = g.div[AX_BLK].d, NM = g.div[AX_MBT].d, TS = NB * NM;
    const uint32_t t_first = first / TS;
    const uint32_t n_items = ((first + count - 1) / TS - t_first + 1) * NM;
    const uint32_t last = first + count;
    for (uint32_t u = blockIdx.x * kBlock + threadIdx.x; u < n_items; u += gridDim.x * kBlock) {
        const uint32_t hi = t_first + u / NM, m_digit = u % NM;
        const uint32_t row0 = hi * TS + m_digit;                  // the row with kv_block digit 0
        // none of this item's rows inside [first, last)?  (only at the ragged ends)
        if (row0 + (NB - 1) * NM < first || row0 >= last) continue;
        const Candidate c = decode_index(s, g, row0);
        const Coef cf = make_coef(s.models[c.model], c.kn.p, c.kn.wbits);
        const HwRecip hw = s.hw[c.hw];
        const PrefillPlan plan = make_prefill_plan(c.kn.b, c.kn.s_in, c.kn.mbt, recip_up(1.0 / (double)c.kn.s_in),
                                                   recip_up(1.0 / (double)c.kn.mbt));
        ExtremeK<false> lo_p, lo_b;
        ExtremeK<true> hi_p, hi_b;
        lo_p.init(); hi_p.init(); lo_b.init(); hi_b.init();
        double sum_p = 0.0, sum_b = 0.0;
        auto sample = [&](uint32_t e, double &tp, double &tb) {
            const TimeCoef tc = make_time_coef(cf, hw.r_peak * s_rec[e], hw.r_bw * s_reb[e], hw.r_link, hw.lat);
            tp = prefill_time_plan<ADDITIVE>(tc, plan, c.kn.b);
            tb = tp + decode_time_fast<ADDITIVE>(tc, c.kn.b, c.kn.s_in, c.kn.s_out - 1);
            sum_p += tp;
            sum_b += tb;
        };
        // Whole groups of eight samples are sorted once (shared by the list of the smallest and the list of
        // the largest) and merged into the lists: 12.5 instead of 28 minimum / maximum operations per sample
        // and metric.  The eight evaluations of a group are unrolled: they are independent, which gives the one
        // or two waves a SIMD holds something to issue while an earlier result is on its way (0.55 against
        // 0.62 ms with the group's samples parked in LDS and the evaluation not unrolled).
        uint32_t e = 0;
        for (; e + kSweepGroup <= n_eff; e += kSweepGroup) {
            double a[kSweepGroup], bb[kSweepGroup];
#pragma unroll
            for (int q = 0; q < kSweepGroup; ++q) sample(e + q, a[q], bb[q]);
            sort_group(a);
            lo_p.merge(a);
            hi_p.merge(a);
            sort_group(bb);
            lo_b.merge(bb);
            hi_b.merge(bb);
        }
        for (; e < n_eff; ++e) {
            double tp, tb;
            sample(e, tp, tb);
            lo_p.push(tp); hi_p.push(tp);
            lo_b.push(tb); hi_b.push(tb);
        }
        const double mean_p = sum_p / (double)n_eff, mean_b = sum_b / (double)n_eff;
        const double p10_p = lo_p.at(r_lo), p90_p = hi_p.at(r_hi), p10_b = lo_b.at(r_lo), p90_b = hi_b.at(r_hi);
        const double cost = cost_of(c.kn, mean_b);
        for (uint32_t k = 0; k < NB; ++k) {
            const uint32_t row = row0 + k * NM;
            if (row < first || row >= last) continue;
            const uint32_t i = row - first;
            if (out.ttft_mean) out.ttft_mean[i] = mean_p;
            if (out.ttft_p10) out.ttft_p10[i] = p10_p;
            if (out.ttft_p90) out.ttft_p90[i] = p90_p;
            if (out.t_batch_mean) out.t_batch_mean[i] = mean_b;
            if (out.t_batch_p10) out.t_batch_p10[i] = p10_b;
            if (out.t_batch_p90) out.t_batch_p90[i] = p90_b;
            if (out.cost) out.cost[i] = cost;
            if (out.b_max || out.feasible) {
                const MemResult mem = memory_check(cf, hw.cap, c.kn.b, c.kn.s_in, c.kn.s_out, s.axis[AX_BLK][k]);
                if (out.b_max) out.b_max[i] = mem.b_max;
                if (out.feasible) out.feasible[i] = mem.feasible ? 1 : 0;
            }
        }
    }
}

// Cluster-level columns under a GPU budget (one index per lane; not on the timed path).
template <bool ADDITIVE>
__global__ __launch_bounds__(kBlock) void eval_extras_kernel(GridDesc g, const DevTables *__restrict__ tab,
                                                             uint32_t first, uint32_t count, uint32_t n_gpus,
                                                             guide_extras out) {
    __shared__ GridLds s;
    stage_grid_tables(s, g, tab);
    __syncthreads();
    for (uint32_t i = blockIdx.x * kBlock + threadIdx.x; i < count; i += gridDim.x * kBlock) {
        const Candidate c = decode_index(s, g, first + i);
        const HwRecip hw = s.hw[c.hw];
        const Coef cf = make_coef(s.models[c.model], c.kn.p, c.kn.wbits);
        const uint32_t dp = n_gpus / c.kn.p;
        const double n = (double)(c.kn.s_out - 1);
        double tok_s = 0.0, tok_s1 = 0.0;
        if (c.kn.s_out > 1 && (out.cluster_tok_s || out.paper_tok_s)) {
            const TimeCoef tc = make_time_coef(cf, hw.r_peak, hw.r_bw, hw.r_link, hw.lat);
            tok_s = (double)c.kn.b * n / decode_time<ADDITIVE>(tc, c.kn.b, c.kn.s_in, c.kn.s_out - 1);
            if (out.paper_tok_s) {
                const Coef c1 = make_coef(s.models[c.model], 1u, c.kn.wbits);      // the same candidate on one GPU
                const TimeCoef t1 = make_time_coef(c1, hw.r_peak, hw.r_bw, hw.r_link, hw.lat);
                tok_s1 = (double)c.kn.b * n / decode_time<ADDITIVE>(t1, c.kn.b, c.kn.s_in, c.kn.s_out - 1);
            }
        }
        const double c_avail = hw.cap - cf.w_gpu;
        const double q = floor(c_avail / ((double)c.kn.b * cf.kv_tok));
        const uint32_t s_max = !(c_avail > 0.0) ? 0u : (q >= 4294967295.0 ? 4294967295u : (uint32_t)q);
        if (out.s_max) out.s_max[i] = s_max;
        if (out.dp_max) out.dp_max[i] = dp;
        const MemResult m = memory_check(cf, hw.cap, c.kn.b, c.kn.s_in, c.kn.s_out, c.kn.blk);
        if (out.max_parallelism) out.max_parallelism[i] = (uint64_t)dp * (uint64_t)m.b_max;
        if (out.b_adj) out.b_adj[i] = c.kn.b < m.b_max ? c.kn.b : m.b_max;
        const bool long_prompt = c.kn.s_in > c.kn.mbt;
        if (out.n_sub_batches) {
            uint32_t split = c.kn.mbt / c.kn.s_in;                    // prompts per pass (0 for a long prompt)
            split = split < c.kn.b ? split : c.kn.b;
            out.n_sub_batches[i] = long_prompt ? c.kn.b : (c.kn.b + split - 1) / split;
        }
        if (out.n_segments) out.n_segments[i] = long_prompt ? (c.kn.s_in - 1) / c.kn.mbt + 1 : 1u;
        if (out.s_adj) {
            const uint32_t len = c.kn.s_in + c.kn.s_out;              // both below 2^31
            out.s_adj[i] = len < s_max ? len : s_max;
        }
        if (out.b_max_kept || out.feasible_kept || out.s_max_kept) {
            // a KV-cache reduction that keeps the fraction kv_keep of every request's entries
            const double keep = out.kv_keep == 0.0 ? 1.0 : out.kv_keep;
            const uint32_t len = c.kn.s_in + c.kn.s_out;
            const uint64_t kept = (uint64_t)ceil(keep * (double)len);
            const uint64_t tok_req = (kept + c.kn.blk - 1) / c.kn.blk * c.kn.blk;
            const double kv_req = (double)tok_req * cf.kv_tok;
            const bool room = c_avail > 0.0;
            const double qb = floor(c_avail / kv_req), qs = floor(q / keep);
            if (out.b_max_kept) out.b_max_kept[i] = !room ? 0u : (qb >= 4294967295.0 ? 4294967295u : (uint32_t)qb);
            if (out.feasible_kept) out.feasible_kept[i] = (room && (double)c.kn.b * kv_req <= c_avail) ? 1 : 0;
            if (out.s_max_kept) out.s_max_kept[i] = !room ? 0u : (qs >= 4294967295.0 ? 4294967295u : (uint32_t)qs);
        }
        if (out.cluster_tok_s) out.cluster_tok_s[i] = (double)dp * tok_s;
        if (out.paper_tok_s)
            out.paper_tok_s[i] = ((double)dp * (double)c.kn.p) * tok_s1 / (1.0 + log2((double)c.kn.p));
    }
}

static uint32_t blocks_for(uint32_t count) {
    const uint32_t need = (count + kBlock - 1) / kBlock;
    const uint32_t cap = device_cus() * 8;
    return need < cap ? need : cap;
}

static uint32_t tile_blocks(uint32_t first, uint32_t count, uint32_t ts) {
    const uint32_t n_tiles = (first + count - 1) / ts - first / ts + 1;
    // two persistent blocks per compute unit: every wave loops over several batches of 64 tiles, so the
    // stores of one batch overlap the arithmetic of the next (measured best among 1..8 blocks per CU)
    // (every block writes one top-k partial when a top-k is folded in)
    uint32_t cap = 2 * device_cus();
    cap = cap < kSelBlocks ? cap : kSelBlocks;
    const uint32_t need = (n_tiles + kBlock - 1) / kBlock;
    return need < cap ? need : cap;
}

// Rows sampled for a Pareto selection over the evaluated rows.
constexpr uint32_t kSampleRows = 16384;
constexpr uint64_t kStreamBytes = 64ull << 20;      // twice the 8 x 4 MB of L2: 8-byte columns that together reach it are streamed
constexpr uint32_t kRiderBlocks = kSampleRows / kBlock;     // sample blocks appended to a plain evaluation
static_assert(kRiderBlocks == kSampleBlocks, "the scratch holds one sample front per sample block");

template <bool ADDITIVE, int NB, int NM>
static void launch_tile(const GridDesc &g, const DevTables *tab, const void *tile_tables, uint32_t first,
                        uint32_t count, double re_c, double re_b, const guide_metrics &out, const FusedSelect *fs,
                        hipStream_t stream, LaunchTiming tm) {
    // fs: a top-k folded into the evaluation (the FUSED kernel) and / or rider_blocks extra blocks that take the
    // row sample of a Pareto selection
    const FusedSelect sel = fs ? *fs : FusedSelect{};
    const dim3 grid(tile_blocks(first, count, NB * NM) + sel.rider_blocks), block(kBlock);
    const TileLds *tables = (const TileLds *)tile_tables;
    // Columns that together are larger than twice the chip's L2 are stored with the streaming hint: their lines
    // would not survive in L2 until a reader comes anyway, and not keeping them there leaves the stores of the
    // launch more room (20M rows: 163 - 166 us against 178 - 179 us; 1.9M rows inside an evaluate-and-select step:
    // 17.4 against 17.8 us, the filter pass after it 13.4 against 13.1 us; smaller outputs stay cached for their readers).
    // (a kernel of its own: a run-time choice between the two kinds of store compiles to the plain one)
    const uint32_t n_f64 = (out.t_prefill ? 1u : 0u) + (out.t_decode ? 1u : 0u) + (out.t_batch ? 1u : 0u) +
                           (out.decode_tok_s ? 1u : 0u) + (out.cost ? 1u : 0u);
    const bool stream_stores = (uint64_t)count * 8 * n_f64 >= kStreamBytes;
    auto launch = [&](auto kernel) {
        // with timing events the launch goes through the extended call, which attaches them to the dispatch
        if (tm.start)
            hipExtLaunchKernelGGL(kernel, grid, block, 0, stream, tm.start, tm.stop, 0, g, tab, first, count, re_c, re_b, out,
                                  sel, tables);
        else
            hipLaunchKernelGGL(kernel, grid, block, 0, stream, g, tab, first, count, re_c, re_b, out, sel, tables);
    };
    if (sel.topk) launch(eval_tile_kernel<ADDITIVE, NB, NM, true, false>);
    else if (stream_stores) launch(eval_tile_kernel<ADDITIVE, NB, NM, false, true>);
    else launch(eval_tile_kernel<ADDITIVE, NB, NM, false, false>);
}

// Tile shapes with a compiled kernel (up to four values on each of the two fastest axes); other grids take the
// one-index-per-lane kernel.
#define GUIDE_TILE_SHAPES(X)                                                                     \
    X(2, 3) X(1, 1) X(1, 2) X(1, 3) X(1, 4) X(2, 1) X(2, 2) X(2, 4) X(3, 1) X(3, 2) X(3, 3) X(3, 4) \
    X(4, 1) X(4, 2) X(4, 3) X(4, 4)

template <bool ADDITIVE>
static bool dispatch_tile(const GridDesc &g, const DevTables *tab, const void *tile_tables, uint32_t first,
                          uint32_t count, double re_c, double re_b, const guide_metrics &out, const FusedSelect *fs,
                          hipStream_t stream, uint32_t *n_blocks, LaunchTiming tm) {
    const uint32_t nb = g.div[AX_BLK].d, nm = g.div[AX_MBT].d;
#define GUIDE_TILE(NB, NM)                                                                   \
    if (nb == NB && nm == NM) {                                                              \
        launch_tile<ADDITIVE, NB, NM>(g, tab, tile_tables, first, count, re_c, re_b, out, fs, stream, tm); \
        if (n_blocks) *n_blocks = tile_blocks(first, count, NB * NM);                        \
        return true;                                                                         \
    }
    GUIDE_TILE_SHAPES(GUIDE_TILE)
#undef GUIDE_TILE
    return false;
}

bool eval_grid_can_fuse(const GridDesc &g) {
    const uint32_t nb = g.div[AX_BLK].d, nm = g.div[AX_MBT].d;
#define GUIDE_TILE(NB, NM) if (nb == NB && nm == NM) return true;
    GUIDE_TILE_SHAPES(GUIDE_TILE)
#undef GUIDE_TILE
    return false;
}

// The tile kernels deal batches of kBlock tiles (kBlock * NB * NM consecutive rows) to their blocks round robin.
uint32_t eval_grid_row_chunk(const GridDesc &g) {
    return eval_grid_can_fuse(g) ? (uint32_t)kBlock * g.div[AX_BLK].d * g.div[AX_MBT].d : 0u;
}

size_t tile_tables_bytes() { return sizeof(TileLds); }

hipError_t launch_tile_tables(const GridDesc &g, const DevTables *tab, void *tile_tables, hipStream_t stream) {
    hipLaunchKernelGGL(tile_tables_kernel, dim3(1), dim3(kBlock), 0, stream, g, tab, (TileLds *)tile_tables);
    return hipGetLastError();
}

hipError_t launch_eval_grid_fused(const GridDesc &g, const DevTables *tab, const void *tile_tables, uint32_t first,
                                  uint32_t count, double e_c, double e_b, bool additive, const guide_metrics &out,
                                  const FusedSelect &fs, hipStream_t stream, uint32_t *n_blocks, LaunchTiming tm) {
    const double re_c = 1.0 / e_c, re_b = 1.0 / e_b;
    FusedSelect sel = fs;
    sel.rider_blocks = fs.pareto ? kRiderBlocks : 0u;
    const bool done =
        additive ? dispatch_tile<true>(g, tab, tile_tables, first, count, re_c, re_b, out, &sel, stream, n_blocks, tm)
                 : dispatch_tile<false>(g, tab, tile_tables, first, count, re_c, re_b, out, &sel, stream, n_blocks, tm);
    return done ? hipGetLastError() : hipErrorNotSupported;
}

hipError_t launch_eval_grid(const GridDesc &g, const DevTables *tab, const void *tile_tables, uint32_t first,
                            uint32_t count, double e_c, double e_b, bool additive, const guide_metrics &out,
                            hipStream_t stream, LaunchTiming tm, const FusedSelect *sample, bool *sampled) {
    const dim3 grid(blocks_for(count)), block(kBlock);
    const double re_c = 1.0 / e_c, re_b = 1.0 / e_b;
    FusedSelect rider;
    const FusedSelect *fs = nullptr;
    if (sampled) *sampled = false;
    if (sample && sampled && eval_grid_can_fuse(g)) {
        rider = *sample;
        rider.topk = 0;
        rider.rider_blocks = kRiderBlocks;
        fs = &rider;
        *sampled = true;
    }
    if (additive ? dispatch_tile<true>(g, tab, tile_tables, first, count, re_c, re_b, out, fs, stream, nullptr, tm)
                 : dispatch_tile<false>(g, tab, tile_tables, first, count, re_c, re_b, out, fs, stream, nullptr, tm))
        return hipGetLastError();
    if (additive && tm.start)
        hipExtLaunchKernelGGL(eval_grid_kernel<true>, grid, block, 0, stream, tm.start, tm.stop, 0, g, tab, first, count,
                              re_c, re_b, out);
    else if (additive)
        hipLaunchKernelGGL(eval_grid_kernel<true>, grid, block, 0, stream, g, tab, first, count, re_c, re_b, out);
    else if (tm.start)
        hipExtLaunchKernelGGL(eval_grid_kernel<false>, grid, block, 0, stream, tm.start, tm.stop, 0, g, tab, first, count,
                              re_c, re_b, out);
    else
        hipLaunchKernelGGL(eval_grid_kernel<false>, grid, block, 0, stream, g, tab, first, count, re_c, re_b, out);
    return hipGetLastError();
}

hipError_t launch_eval_extras(const GridDesc &g, const DevTables *tab, uint32_t first, uint32_t count, uint32_t n_gpus,
                              bool additive, const guide_extras &out, hipStream_t stream) {
    const dim3 grid(blocks_for(count)), block(kBlock);
    if (additive)
        hipLaunchKernelGGL(eval_extras_kernel<true>, grid, block, 0, stream, g, tab, first, count, n_gpus, out);
    else
        hipLaunchKernelGGL(eval_extras_kernel<false>, grid, block, 0, stream, g, tab, first, count, n_gpus, out);
    return hipGetLastError();
}

hipError_t launch_eval_sweep(const GridDesc &g, const DevTables *tab, uint32_t first, uint32_t count, uint32_t n_eff,
                             bool additive, const guide_stats &out, hipStream_t stream) {
    const uint32_t ts = g.div[AX_BLK].d * g.div[AX_MBT].d;
    const uint32_t n_items = ((first + count - 1) / ts - first / ts + 1) * g.div[AX_MBT].d;
    const dim3 grid(blocks_for(n_items)), block(kBlock);
    if (additive)
        hipLaunchKernelGGL(eval_sweep_kernel<true>, grid, block, 0, stream, g, tab, first, count, n_eff, out);
    else
        hipLaunchKernelGGL(eval_sweep_kernel<false>, grid, block, 0, stream, g, tab, first, count, n_eff, out);
    return hipGetLastError();
}

}  // namespace guide
