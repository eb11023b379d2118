// Selection kernels: constrained per-group top-k by (objective, row) order and
// the two-objective Pareto front.  Reductions run in registers and across lanes
// in the vector ALU, then through LDS per block, then in a small second pass over
// the block partials.
//
// Paper: the simulator evaluates every configuration and keeps the one(s) with
// the least total time (Simulating Hybrid Parallelism); the engine keeps the top
// three by inference time / throughput (Inference Engine, Step 2).
#include "kernels.hpp"
#include "reduce.hpp"
#include "select_shared.hpp"

#include <hip/hip_ext.h>

#include <cstring>
#include <type_traits>

namespace guide {

namespace {

constexpr int kWaves = kBlock / kWave;

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

// All loads of a row are issued unconditionally (index clamped when the row is
// past the end) and nothing is computed from them here, so that many rows can be
// in flight while the kernel does other work; row_of() turns the loaded values
// into the row's coordinates and its filter verdict.
// MAXC: constraint columns the kernel variant can hold (n_con <= MAXC); variants with fewer keep
// fewer registers busy per row in flight.
template <uint32_t MAXC>
struct RawRow {
    double x, y;
    double c[MAXC ? MAXC : 1];
    uint8_t fe;
    bool valid;
};
struct Row {
    double x, y;
    bool pass;
};
template <bool WITH_Y, uint32_t MAXC>
__device__ inline RawRow<MAXC> load_raw(const double *__restrict__ x, const double *__restrict__ y, const RowFilter &f,
                                        uint32_t i, uint32_t n) {
    RawRow<MAXC> r;
    r.valid = i < n;
    const uint32_t j = r.valid ? i : 0;
    r.x = x[j];
    r.y = WITH_Y ? y[j] : 0.0;
    r.fe = f.feasible ? f.feasible[j] : (uint8_t)1;
#pragma unroll
    for (uint32_t k = 0; k < MAXC; ++k) r.c[k] = k < f.n_con ? f.col[k][j] : 0.0;
    return r;
}
template <bool WITH_Y, uint32_t MAXC>
__device__ inline Row row_of(const RawRow<MAXC> &w, const RowFilter &f) {
    bool ok = w.valid && w.fe != 0 && (w.x == w.x) && (!WITH_Y || w.y == w.y);
#pragma unroll
    for (uint32_t k = 0; k < MAXC; ++k)
        if (k < f.n_con) ok = ok && (w.c[k] <= f.cap[k]);
    return Row{w.x, w.y, ok};
}
template <bool WITH_Y, uint32_t MAXC>
__device__ inline Row load_row(const double *__restrict__ x, const double *__restrict__ y, const RowFilter &f,
                               uint32_t i, uint32_t n) {
    return row_of<WITH_Y, MAXC>(load_raw<WITH_Y, MAXC>(x, y, f, i, n), f);
}
// Launches fn.template operator()<MAXC>() for the least supported MAXC >= n_con.
template <typename F>
void with_max_constraints(uint32_t n_con, F &&fn) {
    if (n_con == 0) fn(std::integral_constant<uint32_t, 0>{});
    else if (n_con == 1) fn(std::integral_constant<uint32_t, 1>{});
    else fn(std::integral_constant<uint32_t, GUIDE_MAX_CONSTRAINTS>{});
}

// Rows are dealt to blocks in chunks of `chunk` rows (a multiple of kBlock): chunk c goes to block c % gridDim.x.
// The hardware deals blocks to the dies' L2 caches round robin, so with a grid that is a multiple of the number of
// dies, chunk c is read through the same L2 as by any other kernel that deals the same chunks the same way -- in
// particular the evaluation kernel that writes them, which then finds no copies of its lines in other L2s.
// A block walks its chunks in batches of kBlock * U rows (the last batch of a chunk may be partial), U = rows per
// thread in flight: 8, or 6 when that divides the chunk evenly and 8 does not.
constexpr uint32_t kUnroll = 8;
constexpr uint32_t kDefaultChunk = kBlock * kUnroll;
template <uint32_t U>
struct ChunkWalk {
    uint32_t chunk, n, n_blocks, c;
    uint64_t base, end;             // current batch starts at `base`; its chunk ends at `end` (exclusive)
    __device__ ChunkWalk(uint32_t chunk_, uint32_t n_, uint32_t n_blocks_)
        : chunk(chunk_), n(n_), n_blocks(n_blocks_), c(blockIdx.x) { enter(); }
    __device__ void enter() {
        base = (uint64_t)c * chunk;
        end = base + chunk < n ? base + chunk : n;
    }
    __device__ bool live() const { return base < n; }
    __device__ void next() {
        base += kBlock * U;
        if (base >= end) {
            c += n_blocks;
            enter();
        }
    }
};

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

// Blocks of a streaming pass over n rows.  Top-k passes: up to four per compute unit.  The Pareto filter pass:
// three per compute unit -- every block loads a 32 KB table of sample rows and ends with a block-level top-k
// merge, which with more blocks costs more than the extra blocks hide (1.9M rows in chunks of 1536: 13.8 us with
// 768 blocks, 14.5 with 1024, 15.0 with 624, 15.1 - 15.6 with 512, 16.2 with 416).
uint32_t blocks_for(uint64_t n) {
    uint64_t need = (n + kBlock - 1) / kBlock;
    if (need == 0) need = 1;
    return (uint32_t)(need < kSelBlocks ? need : kSelBlocks);
}
uint32_t pareto_blocks(uint64_t n) {
    uint64_t need = (n + kBlock - 1) / kBlock, cap = 3 * (uint64_t)device_cus();
    if (need == 0) need = 1;
    cap = cap < kSelBlocks ? cap : kSelBlocks;
    return (uint32_t)(need < cap ? need : cap);
}

// ------------------------------------------------------- top-k, one group

// Independent work of another selection that rides along with a launch as extra blocks, so that it
// does not pay for a launch of its own.  SampleRider: the row sample of a Pareto selection
// (kSampleBlocks blocks after the host kernel's own).  MergeRider: the merge of top-k block partials
// (one block).  n_blocks = 0 / on = 0: none.
struct SampleRider {
    uint32_t on;
    const double *x, *y;
    RowFilter f;
    SelectScratch *sc;
};
struct MergeRider {
    Top1Ws w;
    uint32_t n_blocks, k, K;       // K: pairs per block partial (1 .. 4)
    uint64_t *out_idx;
    double *out_val;
    uint64_t *out_cnt;
};
__device__ void pareto_prepare_body(uint32_t block, const double *__restrict__ x, const double *__restrict__ y,
                                    const RowFilter &f, uint32_t n, SelectScratch *sc);

// One pass over the rows: every lane keeps its K best, the block merges them.  Blocks
// [0, n_row_blocks) take the rows.
template <int K, uint32_t MAXC, uint32_t U>
__global__ __launch_bounds__(kBlock) void topk_pass_kernel(const double *__restrict__ obj, RowFilter f, uint32_t n,
                                                           Top1Ws w, uint32_t n_row_blocks, SampleRider sample,
                                                           uint32_t chunk) {
    if (blockIdx.x >= n_row_blocks) {
        pareto_prepare_body(blockIdx.x - n_row_blocks, sample.x, sample.y, sample.f, n, sample.sc);
        return;
    }
    __shared__ Pair s_pairs[kWaves][K];
    __shared__ uint64_t s_cnt[kWaves];
    TopList<K> l;
    l.init();
    uint32_t cnt = 0;                                   // rows of one lane: fewer than 2^32
    for (ChunkWalk<U> cw(chunk, n, n_row_blocks); cw.live(); cw.next()) {
        const uint32_t base = (uint32_t)cw.base + threadIdx.x, lim = (uint32_t)cw.end;
        Row r[U];
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) r[u] = load_row<false, MAXC>(obj, nullptr, f, base + u * kBlock, lim);
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            if (r[u].pass) {
                ++cnt;
                l.insert_ascending(Pair{key_of(r[u].x), base + u * kBlock});
            }
        }
    }
    const uint32_t wave_cnt = wave_sum(cnt);             // a wave's rows: fewer than 2^32 as well
    if (threadIdx.x % kWave == 0) s_cnt[threadIdx.x / kWave] = wave_cnt;
    block_topk<K, kWaves>(l, s_pairs, [&](int r, const Pair &p) {
        w.key[(size_t)blockIdx.x * K + r] = p.key;
        w.idx[(size_t)blockIdx.x * K + r] = p.idx;
    });                                                 // (contains the barrier that publishes s_cnt)
    if (threadIdx.x == 0) {
        uint64_t c = 0;
        for (int wv = 0; wv < kWaves; ++wv) c += s_cnt[wv];
        w.cnt[blockIdx.x] = c;
    }
}

// One block of NT threads: the K least of the block partials, and the total count.
constexpr uint32_t kMergeThreads = 512;
template <int K, uint32_t NT>
__device__ inline void topk_merge_body(Top1Ws w, uint32_t n_blocks, uint32_t k, uint64_t *out_idx, double *out_val,
                                       uint64_t *out_cnt) {
    constexpr int kNW = NT / kWave;
    __shared__ Pair s_pairs[kNW][K];
    __shared__ uint64_t s_cnt[kNW];
    constexpr uint32_t kPer = kSelBlocks * K / NT;       // all loads first: one memory latency
    Pair c[kPer];
#pragma unroll
    for (uint32_t q = 0; q < kPer; ++q) {
        const uint32_t i = q * NT + threadIdx.x;
        c[q] = i < n_blocks * K ? Pair{w.key[i], w.idx[i]} : Pair{kNone, kNone};
    }
    uint64_t pc[kSelBlocks / NT];
#pragma unroll
    for (uint32_t q = 0; q < kSelBlocks / NT; ++q) {
        const uint32_t i = q * NT + threadIdx.x;
        pc[q] = i < n_blocks ? w.cnt[i] : 0;
    }
    TopList<K> l;
    l.init();
    uint64_t cnt = 0;
#pragma unroll
    for (uint32_t q = 0; q < kPer; ++q) l.insert(c[q]);
#pragma unroll
    for (uint32_t q = 0; q < kSelBlocks / NT; ++q) cnt += pc[q];
    for (int off = kWave / 2; off > 0; off >>= 1) cnt += __shfl_xor(cnt, off, kWave);
    if (threadIdx.x % kWave == 0) s_cnt[threadIdx.x / kWave] = cnt;
    block_topk<K, kNW>(l, s_pairs, [&](int r, const Pair &p) {
        if ((uint32_t)r < k) {
            out_idx[r] = p.idx;
            out_val[r] = p.idx == kNone ? INFINITY : value_of(p.key);
        }
    });
    if (threadIdx.x == 0) {
        uint64_t t = 0;
        for (int wv = 0; wv < kNW; ++wv) t += s_cnt[wv];
        out_cnt[0] = t;
    }
}

template <int K>
__global__ __launch_bounds__(kMergeThreads) void topk_merge_kernel(Top1Ws w, uint32_t n_blocks, uint32_t k,
                                                                   uint64_t *out_idx, double *out_val, uint64_t *out_cnt) {
    topk_merge_body<K, kMergeThreads>(w, n_blocks, k, out_idx, out_val, out_cnt);
}


// ------------------------------------------------------- top-k, with groups

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
// group's previous pick; round 0 also counts passing rows.  Candidates of one
// group meet in per-wave LDS slots (slot_update).
__global__ __launch_bounds__(kBlock) void topk_round_kernel(const double *__restrict__ obj, RowFilter f,
                                                            const uint32_t *__restrict__ group, uint32_t G,
                                                            uint32_t n, uint32_t round, TopkWs w) {
    __shared__ uint64_t s_key[kWaves][GUIDE_MAX_GROUPS], s_idx[kWaves][GUIDE_MAX_GROUPS];
    __shared__ uint32_t s_cnt[kWaves][GUIDE_MAX_GROUPS];
    const int wave = threadIdx.x / kWave;
    for (uint32_t i = threadIdx.x; i < kWaves * GUIDE_MAX_GROUPS; i += kBlock) {
        (&s_key[0][0])[i] = kNone;
        (&s_idx[0][0])[i] = kNone;
        (&s_cnt[0][0])[i] = 0;
    }
    __syncthreads();
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
            g = group[i];
            ok = (x == x) && g < G && row_passes(f, i);
        }
        Pair p = {kNone, kNone};
        if (ok) {
            p.key = key_of(x);
            p.idx = i;
            if (round == 0) atomicAdd(&s_cnt[wave][g], 1u);
            if (round > 0) {
                const Pair after = {w.after_key[g], w.after_idx[g]};
                ok = less_than(after, p);
            }
        }
        slot_update(s_key[wave], s_idx[wave], g, ok, p);
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
    __shared__ uint64_t s_key[kWaves], s_idx[kWaves], s_cnt[kWaves];
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
        for (int wv = 1; wv < kWaves; ++wv) {
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
//
// Three launches.  The first can ride along with a top-k pass or with the kernel that produces the
// columns; a top-k over the same columns can ride along with the second, and a top-k merge with the last.
// Sample: kSampleBlocks blocks take a scattered sample of rows.  It fixes the stretch of x that the bins
// slice (kBins equal slices of key space, clamped at both ends, so a lower bin means a strictly smaller x),
// and every wave hands over the front of its sample rows.  The block that takes sample 0 also resets the
// counters that the next two kernels accumulate into.
// Filter: every block bins the handed-over sample rows (least y per bin, exclusive prefix-min) and keeps a
// row when no sample row of a strictly lower bin has a y at or below its own.  The kept rows contain the
// front, and every other kept row is dominated by a kept one.  Kept rows are appended as (row, keys).
// Finish: kept rows are binned; those that a kept row of a strictly lower bin dominates (least y per bin
// over the kept rows, exclusive prefix-min) or that their own bin's representative dominates are dropped,
// the rest are grouped by bin and tested exactly inside their bin, and front members are written at (front
// members of lower bins) + (rank inside the bin), which orders the output by (x, y, row).  One block does
// this in LDS for up to kStage kept rows; more are shared out among kLargeParts blocks by runs of bins.

constexpr uint32_t kStage = 4096;        // survivors whose records the finishing block holds in LDS
constexpr uint32_t kFinishThreads = 1024;

// Caller workspace of the Pareto path.
struct ParetoWs {
    uint64_t *skx, *sky;  // [n]: keys of surviving rows
    uint32_t *surv;       // [n]: surviving rows, arbitrary order
    // large-front path only:
    uint32_t *staged;     // [n]: per part of the front, from its first survivor slot on: its front members' rows in order
    uint32_t *grouped;    // [n]: positions into surv, grouped by bin (parts whose survivors do not fit LDS)
    uint8_t *on_front;    // [n]: flag per grouped survivor (the same parts)
    uint8_t *dead;        // [n]: flag per survivor slot: a survivor of a lower bin dominates it
};
size_t pareto_ws_bytes(uint64_t n) { return (size_t)n * (8 + 8 + 4 + 4 + 4 + 1 + 1) + 256; }
ParetoWs pareto_ws(void *ws, uint64_t n) {
    ParetoWs w;
    w.skx = (uint64_t *)ws;
    w.sky = w.skx + n;
    w.surv = (uint32_t *)(w.sky + n);
    w.staged = w.surv + n;
    w.grouped = w.staged + n;
    w.on_front = (uint8_t *)(w.grouped + n);
    w.dead = w.on_front + n;
    return w;
}

struct Binning {
    uint64_t lo;
    uint32_t shift;
    __device__ uint32_t operator()(uint64_t kx) const {
        if (kx <= lo) return 0;
        const uint64_t b = (kx - lo) >> shift;
        return b < kBins ? (uint32_t)b : kBins - 1;
    }
};
__device__ inline Binning binning_of(uint64_t lo, uint64_t hi) {
    Binning b;
    b.lo = lo;
    const uint64_t span = hi - lo;
    // least shift with (span >> shift) < kBins
    const uint32_t bits = span ? 64u - (uint32_t)__builtin_clzll(span) : 0u;   // span < 2^bits
    constexpr uint32_t kBinBits = 12;
    static_assert((1u << kBinBits) == kBins, "kBins is a power of two");
    b.shift = bits > kBinBits ? bits - kBinBits : 0u;
    return b;
}

// Range that the bins slice, from a strided sample of rows: low end = least x of
// passing sample rows, high end = x of the sample row with the least y (rows
// beyond it are dominated by that row unless their y is smaller still; they share
// the last bin).  Any monotone binning is correct -- the sample only decides how
// finely the interesting stretch of x is resolved.
__device__ void pareto_prepare_body(uint32_t block, const double *__restrict__ x, const double *__restrict__ y,
                                    const RowFilter &f, uint32_t n, SelectScratch *sc) {
    __shared__ uint64_t s_lo[kWaves];
    __shared__ Pair s_best[kWaves];
    const uint32_t gid = block * kBlock + threadIdx.x;
    const uint32_t n_samples = kSampleBlocks * kBlock;
    if (gid == 0) sc->counters[0] = sc->counters[1] = 0;         // neutral state for the kernels that follow
    const uint32_t stride = n > n_samples ? n / n_samples : 1;
    const uint32_t k = sample_number(block, kSampleBlocks);
    const Row r = load_row<true, GUIDE_MAX_CONSTRAINTS>(x, y, f, (uint64_t)k * stride < n ? sample_row(k, stride) : n, n);
    uint64_t lo = kNone, kx = 0, ky = 0;
    Pair best = {kNone, kNone};                                     // (y key, x key) of the least y
    if (r.pass) {
        lo = kx = key_of(r.x);
        ky = key_of(r.y);
        best = Pair{ky, kx};
    }
    lo = wave_min(lo);
    best = wave_min(best);
    if (threadIdx.x % kWave == 0) {
        s_lo[threadIdx.x / kWave] = lo;
        s_best[threadIdx.x / kWave] = best;
    }
    store_sample_front(r.pass, kx, ky, sc->sample_front + block * kSampleFrontPer);
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int wv = 1; wv < kWaves; ++wv) {
            lo = s_lo[wv] < lo ? s_lo[wv] : lo;
            best = pair_min(best, s_best[wv]);
        }
        sc->sample_lo[block] = lo;
        sc->sample_best[block] = best;
    }
}
__global__ __launch_bounds__(kBlock) void pareto_prepare_kernel(const double *__restrict__ x,
                                                                const double *__restrict__ y, RowFilter f, uint32_t n,
                                                                SelectScratch *sc) {
    pareto_prepare_body(blockIdx.x, x, y, f, n, sc);
}

// Combines the kSampleBlocks per-block sample partials (the same result in every block): the
// first wave loads them, one per lane, and reduces; s_rng (2 entries) carries the result to
// the other waves.  Contains a block barrier.
__device__ inline Binning sampled_binning(const SelectScratch *sc, uint64_t *s_rng) {
    static_assert(kSampleBlocks == kWave, "one partial per lane of the first wave");
    if (threadIdx.x < kWave) {
        uint64_t lo = wave_min(sc->sample_lo[threadIdx.x]);
        const Pair best = wave_min(sc->sample_best[threadIdx.x]);
        uint64_t hi = best.idx;
        if (lo == kNone || hi < lo) {   // no passing sample row: one slice per 2^52 keys
            lo = 0;
            hi = kNone;
        }
        if (threadIdx.x == 0) {
            s_rng[0] = lo;
            s_rng[1] = hi;
        }
    }
    __syncthreads();
    return binning_of(s_rng[0], s_rng[1]);
}

// kBins-entry tables in LDS that a block scans are stored with one unused slot after every PER
// entries (PER = entries per thread of the scan): thread t's entries then start at slot t * (PER + 1),
// and the lanes of a wave reach different banks when each reads its own j-th entry.
template <uint32_t PER>
__device__ inline uint32_t padded(uint32_t i) { return i + i / PER; }
template <uint32_t PER>
constexpr uint32_t padded_size() { return kBins + kBins / PER + 1; }
constexpr uint32_t kPerPass = kBins / kBlock;             // table entries per thread of a streaming block
constexpr uint32_t kPerFinish = kBins / 1024;             // ... of the finishing block

// Thread t of the NT-thread block owns the kBins / NT consecutive entries v[] of a
// kBins-entry table; returns the minimum over all entries before its first one
// (scan in the wave, wave totals through LDS; one block barrier).
// s_tmp: NT / kWave entries.
template <uint32_t NT>
__device__ inline uint64_t prefix_min_before(const uint64_t (&v)[kBins / NT], uint64_t *s_tmp) {
    constexpr uint32_t per = kBins / NT, nw = NT / kWave;
    const uint32_t t = threadIdx.x, lane = t % kWave, wave = t / kWave;
    uint64_t m = kNone;
#pragma unroll
    for (uint32_t j = 0; j < per; ++j) m = min_u64(m, v[j]);
    const uint64_t inc = wave_scan_min(m);              // inclusive scan of thread minima in the wave
    if (lane == kWave - 1) s_tmp[wave] = inc;
    uint64_t run = __shfl_up(inc, 1, kWave);            // exclusive within the wave
    if (lane == 0) run = kNone;
    __syncthreads();
    for (uint32_t wv = 0; wv < nw; ++wv)
        if (wv < wave) run = min_u64(run, s_tmp[wv]);
    return run;
}

// Exclusive prefix-min over a (padded) kBins-entry table in LDS, in place, by the NT threads of the block.
template <uint32_t NT>
__device__ inline void scan_min_excl(uint64_t *s_io, uint64_t *s_tmp) {
    constexpr uint32_t per = kBins / NT;
    const uint32_t t = threadIdx.x;
    uint64_t v[per];
#pragma unroll
    for (uint32_t j = 0; j < per; ++j) v[j] = s_io[t * (per + 1) + j];
    uint64_t run = prefix_min_before<NT>(v, s_tmp);
#pragma unroll
    for (uint32_t j = 0; j < per; ++j) {
        s_io[t * (per + 1) + j] = run;
        run = min_u64(run, v[j]);
    }
    __syncthreads();
}

// Exclusive prefix-sum over a kBins-entry table, in place, by the NT threads of the block; the total
// goes to entry kBins.  PAD: the table is a padded LDS table; otherwise plain (global memory).
// s_tmp: NT / kWave entries.
template <uint32_t NT, bool PAD>
__device__ inline void scan_sum_excl(uint32_t *io, uint32_t *s_tmp) {
    constexpr uint32_t per = kBins / NT, nw = NT / kWave, pitch = PAD ? per + 1 : per;
    const uint32_t t = threadIdx.x, lane = t % kWave, wave = t / kWave;
    uint32_t v[per], m = 0;
#pragma unroll
    for (uint32_t j = 0; j < per; ++j) {
        v[j] = io[t * pitch + j];
        m += v[j];
    }
    const uint32_t inc = wave_scan_sum(m);
    if (lane == kWave - 1) s_tmp[wave] = inc;
    uint32_t run = inc - m;
    __syncthreads();
    uint32_t total = 0;
    for (uint32_t wv = 0; wv < nw; ++wv) {
        if (wv < wave) run += s_tmp[wv];
        total += s_tmp[wv];
    }
#pragma unroll
    for (uint32_t j = 0; j < per; ++j) {
        io[t * pitch + j] = run;
        run += v[j];
    }
    if (t == 0) io[PAD ? padded<per>(kBins) : kBins] = total;
    __syncthreads();
}

// A top-k selection over the same rows that reads nothing but the Pareto selection's two columns and its
// flag column: the staircase kernel has those values in registers anyway and keeps the per-lane lists
// beside its own work, so the top-k needs no pass of its own.
struct SharedTopk {
    uint32_t obj_is_y;             // objective: 0 = the x column, 1 = the y column
    uint32_t use_feasible;         // rows with flag 0 do not pass
    uint32_t n_con;                // <= 2 constraints, each on x or y
    uint32_t con_is_y[2];
    double cap[2];
    Top1Ws w;                      // block partials, as written by the top-k pass
};

// The filter pass of the three-launch form: the sampling blocks have handed over the front of their sample
// rows (SelectScratch::sample_front); every block bins those few rows in LDS (least y per bin, then its
// exclusive prefix-min) and keeps a row when no sample row of a strictly lower bin has a y at or below its
// own.  Every row of the front is kept, and every other kept row is dominated by a kept one (its
// dominators are themselves dominated by a front row, and domination is transitive).  Kept rows are appended
// as (row, keys), counted per bin, and their least y per bin goes to the global table, whose exclusive
// prefix-min tells the finishing kernel which kept rows a kept row of a lower bin dominates.
// KT: pairs per block partial of a top-k that shares the columns (0 = none), as in the staircase kernel.
template <uint32_t MAXC, int KT, uint32_t U>
__global__ __launch_bounds__(kBlock) void pareto_filter_kernel(const double *__restrict__ x, const double *__restrict__ y,
                                                               RowFilter f, uint32_t n, ParetoWs w, SelectScratch *sc,
                                                               SharedTopk topk, uint32_t chunk) {
    __shared__ uint64_t s_lower[padded_size<kPerPass>()], s_tmp[kWaves], s_rng[2];
    constexpr int KL = KT ? KT : 1;
    constexpr uint32_t kPerSample = kSampleBlocks * kSampleFrontPer / kBlock;
    static_assert(kSampleBlocks * kSampleFrontPer % kBlock == 0, "whole sample rows per thread");
    const int lane = threadIdx.x % kWave;
    TopList<KL> list;
    uint32_t n_pass = 0;                                // rows of one lane: fewer than 2^32
    if (KT) list.init();
    // requested first, and in this order: the sample rows, then the first batch of rows, whose latency
    // overlaps the set-up of the table
    Pair sf[kPerSample];
#pragma unroll
    for (uint32_t j = 0; j < kPerSample; ++j) sf[j] = sc->sample_front[j * kBlock + threadIdx.x];
    RawRow<MAXC> r[U];
    ChunkWalk<U> cw(chunk, n, gridDim.x);
    if (cw.live()) {
#pragma unroll
        for (uint32_t u = 0; u < U; ++u)
            r[u] = load_raw<true, MAXC>(x, y, f, (uint32_t)cw.base + threadIdx.x + u * kBlock, (uint32_t)cw.end);
    }
    for (uint32_t i = threadIdx.x; i < padded_size<kPerPass>(); i += kBlock) s_lower[i] = kNone;
    const Binning bin = sampled_binning(sc, s_rng);     // its barrier also covers the table above
#pragma unroll
    for (uint32_t j = 0; j < kPerSample; ++j)
        if (sf[j].idx != kNone)
            atomicMin((unsigned long long *)&s_lower[padded<kPerPass>(bin(sf[j].idx))], (unsigned long long)sf[j].key);
    __syncthreads();
    scan_min_excl<kBlock>(s_lower, s_tmp);              // least y of the sample rows in strictly lower bins
    // wave-uniform trip count: the ballots below need every lane
    while (cw.live()) {
        const uint32_t base = (uint32_t)cw.base;
        // the next batch is requested before this one is worked on
        RawRow<MAXC> rn[U];
        cw.next();
        const bool more = cw.live();
        if (more) {
#pragma unroll
            for (uint32_t u = 0; u < U; ++u)
                rn[u] = load_raw<true, MAXC>(x, y, f, (uint32_t)cw.base + threadIdx.x + u * kBlock, (uint32_t)cw.end);
        }
        // Kept rows are rare and come in clusters: the wave counts them over the whole batch and appends them
        // with one atomic (a wave that waits for one atomic per row slot waits several memory round trips).
        uint32_t keep_bits = 0, total = 0, before[U];
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            const Row q = row_of<true, MAXC>(r[u], f);
            const bool keep = q.pass && key_of(q.y) < s_lower[padded<kPerPass>(bin(key_of(q.x)))];
            const uint64_t mask = __ballot(keep);
            before[u] = total + (uint32_t)__popcll(mask & ((1ull << lane) - 1));
            total += (uint32_t)__popcll(mask);
            keep_bits |= keep ? 1u << u : 0u;
        }
        if (total) {                                    // wave-uniform
            uint32_t at = 0;
            if (lane == 0) at = atomicAdd(&sc->counters[0], total);
            at = (uint32_t)__builtin_amdgcn_readfirstlane((int)at);
#pragma unroll
            for (uint32_t u = 0; u < U; ++u) {
                if ((keep_bits >> u) & 1u) {
                    const Row q = row_of<true, MAXC>(r[u], f);
                    const uint64_t kx = key_of(q.x), ky = key_of(q.y);
                    const uint32_t slot = at + before[u];
                    w.surv[slot] = base + threadIdx.x + u * kBlock;
                    w.skx[slot] = kx;
                    w.sky[slot] = ky;
                }
            }
        }
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            const uint32_t i = base + threadIdx.x + u * kBlock;
            if (KT) {
                const double obj = topk.obj_is_y ? r[u].y : r[u].x;
                bool ok = r[u].valid && (!topk.use_feasible || r[u].fe != 0) && obj == obj;
#pragma unroll
                for (uint32_t c = 0; c < 2; ++c)
                    if (c < topk.n_con) ok = ok && ((topk.con_is_y[c] ? r[u].y : r[u].x) <= topk.cap[c]);
                if (ok) {
                    ++n_pass;
                    list.insert_ascending(Pair{key_of(obj), (uint64_t)i});
                }
            }
        }
        if (more) {
#pragma unroll
            for (uint32_t u = 0; u < U; ++u) r[u] = rn[u];
        }
    }
    if (KT) {
        __shared__ Pair s_pairs[kWaves][KL];
        __shared__ uint64_t s_cnt[kWaves];
        int my_rank = -1;
        Pair my_pair = {kNone, kNone};
        const uint32_t wave_pass = wave_sum(n_pass);
        if (threadIdx.x % kWave == 0) s_cnt[threadIdx.x / kWave] = wave_pass;
        block_topk<KL, kWaves>(list, s_pairs, [&](int rk, const Pair &p) {
            my_rank = rk;
            my_pair = p;
        });                                             // (contains the barrier that publishes s_cnt)
        if (my_rank >= 0) {
            topk.w.key[(size_t)blockIdx.x * KL + my_rank] = my_pair.key;
            topk.w.idx[(size_t)blockIdx.x * KL + my_rank] = my_pair.idx;
        }
        if (threadIdx.x == 0) {
            uint64_t c = 0;
            for (int wv = 0; wv < kWaves; ++wv) c += s_cnt[wv];
            topk.w.cnt[blockIdx.x] = c;
        }
    }
}

// LDS of the finishing kernel.
constexpr uint16_t kDeadBit = 0x8000;
static_assert(kBins <= kDeadBit, "a bin number and the flag share 16 bits");
struct FinishLds {
    union {
        struct {
            uint32_t off[padded_size<kPerFinish>()];    // first survivor slot per bin (exclusive scan of the bin counts)
            uint32_t foff[padded_size<kPerFinish>()];   // front members per bin, then their exclusive scan
        };
        // before the bins are counted: per bin, the least x among its survivors with the bin's least y
        uint64_t rep[kBins];
    };
    uint32_t cur[kBins];                        // fill level per bin while grouping; then the list of front members
    uint32_t tmp[kFinishThreads / kWave];
    uint64_t tmp64[kFinishThreads / kWave];
    union {
        struct {
            uint64_t kx[kStage], ky[kStage];    // staged survivor records, grouped by bin
        };
        // before anything is staged: per bin, the least y among the survivors of strictly lower bins (padded table)
        uint64_t lower[padded_size<kPerFinish>()];
    };
    uint32_t row[kStage];
    uint16_t bin[kStage];                       // bin of the record; kDeadBit: a survivor of a lower bin dominates it
    uint8_t flag[kStage];
    uint32_t nfront, first, last, is_last;
    uint32_t part_base[kWave], part_lo[kWave], part_cnt[kWave];
    uint64_t rng[2];
};

// The front among `cnt` survivor records staged in LDS, grouped by bin: record i of bin b sits at
// L.off[b] - base + i.  L.foff must be zero and the staging complete (the function starts with a barrier).
// Calls emit(position, row) for every front member, position = its rank by (bin, x, y, row) among the
// front members staged here, and returns their number.
// GROUP lanes per survivor (8 or 1): they share out the members of its bin, four LDS reads in flight each, and
// meet through a wave ballot.  A survivor's test is a chain of dependent LDS reads, so many survivors are kept
// in flight.  Up to 1024 survivors, eight lanes each are fastest (one lane per survivor: one round over all of
// them but longer chains, +1 to +6 us, the fullest bin setting the pace); beyond, one lane each saves more
// rounds (a round over 128 survivors costs about as much as one over 1024) than the chains cost.
template <uint32_t GROUP, typename Emit>
__device__ inline uint32_t staged_front_by(FinishLds &L, uint32_t cnt, uint32_t base, Emit &&emit) {
    constexpr uint32_t P = kPerFinish, group = GROUP, q_step = kFinishThreads / group;
    constexpr uint64_t group_mask = group < 64 ? (1ull << group) - 1 : ~0ull;
    const uint32_t t = threadIdx.x, lane = t % kWave, sub = lane % group, shift = lane - sub;
    __syncthreads();
    const uint32_t cnt_pad = (cnt + q_step - 1) / q_step * q_step;      // wave-uniform trip count for the ballot
    for (uint32_t q = t / group; q < cnt_pad; q += q_step) {
        const bool live = q < cnt;
        const uint64_t kx = live ? L.kx[q] : 0, ky = live ? L.ky[q] : 0;
        const uint32_t bq = live ? L.bin[q] : 0, b = bq & (kDeadBit - 1);
        bool dom = (bq & kDeadBit) != 0;            // then its own bin need not be searched
        const uint32_t beg = live ? L.off[padded<P>(b)] - base : 0, end = live && !dom ? L.off[padded<P>(b + 1)] - base : beg;
        for (uint32_t j = beg + sub; j < end; j += 4 * group) {
            uint64_t jx[4], jy[4];
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u) {      // past the end: the bin's first member once more
                const uint32_t jj = j + u * group < end ? j + u * group : beg;
                jx[u] = L.kx[jj];
                jy[u] = L.ky[jj];
            }
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u)
                dom = dom || (jx[u] <= kx && jy[u] <= ky && (jx[u] < kx || jy[u] < ky));
        }
        const bool dominated = ((__ballot(dom) >> shift) & group_mask) != 0;
        if (live && sub == 0) {
            L.flag[q] = dominated ? 0 : 1;
            if (!dominated) {
                atomicAdd(&L.foff[padded<P>(b)], 1u);
                L.cur[atomicAdd(&L.nfront, 1u)] = q;        // L.cur is free again: list of front members
            }
        }
    }
    __syncthreads();
    scan_sum_excl<kFinishThreads, true>(L.foff, L.tmp);
    const uint32_t nf = L.nfront;
    const uint32_t f_pad = (nf + q_step - 1) / q_step * q_step;          // wave-uniform trip count for the shuffles
    for (uint32_t qf = t / group; qf < f_pad; qf += q_step) {
        const bool live = qf < nf;
        const uint32_t q = live ? L.cur[qf] : 0;
        const uint64_t kx = live ? L.kx[q] : 0, ky = live ? L.ky[q] : 0;
        const uint32_t b = live ? L.bin[q] & (kDeadBit - 1) : 0, i = live ? L.row[q] : 0;
        const uint32_t beg = live ? L.off[padded<P>(b)] - base : 0, end = live ? L.off[padded<P>(b + 1)] - base : 0;
        uint32_t rank = 0;                          // front members of the bin that come before this one
        for (uint32_t j = beg + sub; j < end; j += 4 * group) {
            uint64_t jx[4], jy[4];
            uint32_t jr[4];
            bool on[4];
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u) {
                const uint32_t jj = j + u * group;
                on[u] = jj < end;
                const uint32_t jc = on[u] ? jj : beg;
                on[u] = on[u] && L.flag[jc];
                jx[u] = L.kx[jc];
                jy[u] = L.ky[jc];
                jr[u] = L.row[jc];
            }
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u)
                rank += (on[u] && (jx[u] < kx || (jx[u] == kx && (jy[u] < ky || (jy[u] == ky && jr[u] < i))))) ? 1u : 0u;
        }
        for (uint32_t off = 1; off < group; off <<= 1) rank += __shfl_xor(rank, off, kWave);
        if (live && sub == 0) emit(L.foff[padded<P>(b)] + rank, i);
    }
    return nf;
}
// b_lo .. b_hi: the bins that hold the staged survivors.  One lane per survivor only when there are more than
// 1024 of them and a survivor's bin holds 32 members or fewer on average over the survivors (sum of squared bin
// counts <= 32 * cnt): crowded bins want the eight lanes (400 000 front rows took 2.2 instead of 2.1 ms,
// 1 900 800 took 32.5 instead of 31.2 ms with one lane each), sparse ones the fewer rounds (4 000 front rows:
// 26 instead of 60 us).
template <typename Emit>
__device__ inline uint32_t staged_front(FinishLds &L, uint32_t cnt, uint32_t base, uint32_t b_lo, uint32_t b_hi,
                                        Emit &&emit) {
    if (cnt <= 1024) return staged_front_by<8>(L, cnt, base, emit);     // block-uniform
    constexpr uint32_t P = kPerFinish;
    uint32_t sq = 0;                                    // at most cnt * kStage < 2^32
#pragma unroll
    for (uint32_t q = 0; q < P; ++q) {
        const uint32_t b = q * kFinishThreads + threadIdx.x;
        const uint32_t n = (b >= b_lo && b <= b_hi) ? L.off[padded<P>(b + 1)] - L.off[padded<P>(b)] : 0u;
        sq += n * n;
    }
    sq = wave_sum(sq);
    __syncthreads();                                    // L.tmp may still be read by the scan before
    if (threadIdx.x % kWave == 0) L.tmp[threadIdx.x / kWave] = sq;
    __syncthreads();
    uint32_t total = 0;
    for (uint32_t wv = 0; wv < kFinishThreads / kWave; ++wv) total += L.tmp[wv];
    return total <= 32 * cnt ? staged_front_by<1>(L, cnt, base, emit) : staged_front_by<8>(L, cnt, base, emit);
}

// The same for bins b_lo .. b_hi when their survivors do not fit the staging arrays: the records stay in the
// workspace, reached through w.grouped (already grouped by bin: slots L.off[b_lo] .. L.off[b_hi + 1]), flags
// in w.on_front.
template <typename Emit>
__device__ inline uint32_t unstaged_front(FinishLds &L, const ParetoWs &w, const Binning &bin, uint32_t b_lo, uint32_t b_hi,
                                          Emit &&emit) {
    constexpr uint32_t P = kPerFinish, NT = kFinishThreads, group = 8, q_step = NT / group;
    constexpr uint64_t group_mask = (1ull << group) - 1;
    const uint32_t t = threadIdx.x, lane = t % kWave, sub = lane % group, shift = lane - sub;
    const uint32_t g_lo = L.off[padded<P>(b_lo)], cnt = L.off[padded<P>(b_hi + 1)] - g_lo;
    const uint32_t cnt_pad = (cnt + q_step - 1) / q_step * q_step;       // wave-uniform trip counts
    for (uint32_t k = t / group; k < cnt_pad; k += q_step) {
        const bool live = k < cnt;
        const uint32_t g = g_lo + (live ? k : 0), q = w.grouped[g];
        const uint64_t kx = w.skx[q], ky = w.sky[q];
        const uint32_t b = bin(kx), beg = L.off[padded<P>(b)];
        bool dom = w.dead[q] != 0;                      // then its own bin need not be searched
        const uint32_t end = dom ? beg : L.off[padded<P>(b + 1)];
        for (uint32_t j = beg + sub; j < end; j += 2 * group) {
            const uint32_t j1 = j + group < end ? j + group : beg;       // past the end: the first member again
            const uint32_t q0 = w.grouped[j], q1 = w.grouped[j1];
            const uint64_t x0 = w.skx[q0], y0 = w.sky[q0], x1 = w.skx[q1], y1 = w.sky[q1];
            dom = dom || (x0 <= kx && y0 <= ky && (x0 < kx || y0 < ky)) || (x1 <= kx && y1 <= ky && (x1 < kx || y1 < ky));
        }
        const bool dominated = ((__ballot(dom) >> shift) & group_mask) != 0;
        if (live && sub == 0) {
            w.on_front[g] = dominated ? 0 : 1;
            if (!dominated) atomicAdd(&L.foff[padded<P>(b)], 1u);
        }
    }
    __syncthreads();
    scan_sum_excl<NT, true>(L.foff, L.tmp);
    for (uint32_t k = t / group; k < cnt_pad; k += q_step) {
        const bool live = k < cnt;
        const uint32_t g = g_lo + (live ? k : 0), q = w.grouped[g];
        const bool front = live && w.on_front[g];
        uint32_t rank = 0, b = 0;
        if (front) {
            const uint64_t kx = w.skx[q], ky = w.sky[q];
            b = bin(kx);
            const uint32_t beg = L.off[padded<P>(b)], end = L.off[padded<P>(b + 1)];
            for (uint32_t j = beg + sub; j < end; j += group) {
                if (!w.on_front[j]) continue;
                const uint32_t qj = w.grouped[j];
                const uint64_t jx = w.skx[qj], jy = w.sky[qj];
                if (jx < kx || (jx == kx && (jy < ky || (jy == ky && w.surv[qj] < w.surv[q])))) ++rank;
            }
        }
        for (uint32_t off = 1; off < group; off <<= 1) rank += __shfl_xor(rank, off, kWave);
        if (front && sub == 0) emit(L.foff[padded<P>(b)] + rank, w.surv[q]);
    }
    return L.foff[padded<P>(kBins)];
}

// A front of more than kStage survivors, finished by the n_parts blocks of the launch that call this (part =
// 0 .. n_parts - 1).  Bins are independent until positions in the output are handed out, so each part takes a
// run of consecutive bins that holds about m / n_parts survivors (bin b belongs to part floor(first survivor
// slot of b * n_parts / m)), finds the front members among them, and writes their rows, in order, to the
// workspace from its first survivor slot on.  No part waits for
// another: each ends by taking a ticket, and the part that draws the last one lines the parts' runs up in
// the output.
constexpr uint32_t kLargeParts = 64;                    // blocks that finish a large front (the finishing block is one)
static_assert(kLargeParts <= kWave, "the last part scans the parts' counts in one wave");
static_assert(kLargeParts <= sizeof(SelectScratch::part_cnt) / sizeof(uint32_t), "one scratch entry per part");
__device__ void pareto_large_front(FinishLds &L, const ParetoWs &w, SelectScratch *sc, const Binning &bin, uint32_t m,
                                   uint32_t part, uint32_t n_parts, uint64_t *out_idx, uint64_t capacity,
                                   uint64_t *out_count) {
    constexpr uint32_t P = kPerFinish, NT = kFinishThreads;
    const uint32_t t = threadIdx.x;
    // One pass over all survivors: survivors per bin and the least y per bin, both in LDS (the latter where
    // records are staged afterwards).  Four records are requested at a time.
#pragma unroll
    for (uint32_t q = 0; q < P; ++q) {
        const uint32_t i = q * NT + t;
        L.off[padded<P>(i)] = 0;
        L.foff[padded<P>(i)] = 0;
        L.cur[i] = 0;
    }
    for (uint32_t i = t; i < padded_size<P>(); i += NT) L.lower[i] = kNone;
    if (t == 0) {
        L.first = kBins;
        L.last = 0;
    }
    __syncthreads();
    for (uint32_t q0 = t; q0 < m; q0 += 4 * NT) {
        uint64_t kx[4], ky[4];
#pragma unroll
        for (uint32_t u = 0; u < 4; ++u) {
            const uint32_t q = q0 + u * NT < m ? q0 + u * NT : q0;
            kx[u] = w.skx[q];
            ky[u] = w.sky[q];
        }
#pragma unroll
        for (uint32_t u = 0; u < 4; ++u) {
            if (q0 + u * NT < m) {
                const uint32_t b = padded<P>(bin(kx[u]));
                atomicAdd(&L.off[b], 1u);
                atomicMin((unsigned long long *)&L.lower[b], (unsigned long long)ky[u]);
            }
        }
    }
    __syncthreads();
    scan_sum_excl<NT, true>(L.off, L.tmp);              // entry kBins = m
    scan_min_excl<NT>(L.lower, L.tmp64);                // least y among the survivors of strictly lower bins
#pragma unroll
    for (uint32_t q = 0; q < P; ++q) {
        const uint32_t i = q * NT + t, off = L.off[padded<P>(i)];
        if (L.off[padded<P>(i + 1)] != off && (uint32_t)((uint64_t)off * n_parts / m) == part) {
            atomicMin(&L.first, i);
            atomicMax(&L.last, i);
        }
    }
    __syncthreads();
    const uint32_t b_lo = L.first, b_hi = L.last;       // this part's bins (non-empty ones in between are all its own)
    // Which of the part's survivors a survivor of a lower bin dominates: a second pass, before anything is
    // staged over the table.
    if (b_lo <= b_hi) {
        for (uint32_t q0 = t; q0 < m; q0 += 4 * NT) {
            uint64_t kx[4];
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u) kx[u] = w.skx[q0 + u * NT < m ? q0 + u * NT : q0];
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u) {
                const uint32_t q = q0 + u * NT, b = bin(kx[u]);
                if (q < m && b >= b_lo && b <= b_hi) w.dead[q] = w.sky[q] >= L.lower[padded<P>(b)] ? 1 : 0;
            }
        }
    }
    __syncthreads();
    uint32_t g_lo = 0, n_front = 0;
    if (b_lo <= b_hi) {
        g_lo = L.off[padded<P>(b_lo)];
        auto emit = [&](uint32_t pos, uint32_t row) { w.staged[g_lo + n_front + pos] = row; };
        // In rounds: each takes as many of the part's bins as fit the staging arrays (a single bin that does
        // not fit is finished in the workspace instead).  A part with one round picks its survivors out of
        // one pass over all of them; a part with more first groups its survivors by bin in the workspace, in
        // one such pass, and every round then copies its stretch.  Four keys are requested at a time: the
        // pass is a chain of load latencies otherwise.
        const bool grouped = L.off[padded<P>(b_hi + 1)] - g_lo > kStage;
        if (grouped) {
            for (uint32_t q0 = t; q0 < m; q0 += 4 * NT) {
                uint64_t kx[4];
#pragma unroll
                for (uint32_t u = 0; u < 4; ++u) kx[u] = w.skx[q0 + u * NT < m ? q0 + u * NT : q0];
#pragma unroll
                for (uint32_t u = 0; u < 4; ++u) {
                    const uint32_t q = q0 + u * NT, b = bin(kx[u]);
                    if (q < m && b >= b_lo && b <= b_hi) w.grouped[L.off[padded<P>(b)] + atomicAdd(&L.cur[b], 1u)] = q;
                }
            }
        }
        for (uint32_t r_lo = b_lo; r_lo <= b_hi;) {
            __syncthreads();                            // the previous round is done with the tables
            if (t == 0) {
                L.last = r_lo;
                L.nfront = 0;
            }
            const uint32_t base = L.off[padded<P>(r_lo)];
#pragma unroll
            for (uint32_t q = 0; q < P; ++q) {
                const uint32_t i = q * NT + t;
                L.foff[padded<P>(i)] = 0;
                L.cur[i] = 0;
            }
            __syncthreads();
#pragma unroll
            for (uint32_t q = 0; q < P; ++q) {
                const uint32_t i = q * NT + t;
                if (i > r_lo && i <= b_hi && L.off[padded<P>(i + 1)] - base <= kStage) atomicMax(&L.last, i);
            }
            __syncthreads();
            const uint32_t r_hi = L.last, cnt = L.off[padded<P>(r_hi + 1)] - base;
            uint32_t nf;
            if (cnt <= kStage && grouped) {
                for (uint32_t i = t; i < cnt; i += NT) {
                    const uint32_t q = w.grouped[base + i];
                    const uint64_t kx = w.skx[q];
                    L.kx[i] = kx;
                    L.ky[i] = w.sky[q];
                    L.row[i] = w.surv[q];
                    L.bin[i] = (uint16_t)(bin(kx) | (w.dead[q] ? kDeadBit : 0));
                }
                nf = staged_front(L, cnt, base, r_lo, r_hi, emit);
            } else if (cnt <= kStage) {
                for (uint32_t q0 = t; q0 < m; q0 += 4 * NT) {
                    uint64_t kx[4];
#pragma unroll
                    for (uint32_t u = 0; u < 4; ++u) kx[u] = w.skx[q0 + u * NT < m ? q0 + u * NT : q0];
#pragma unroll
                    for (uint32_t u = 0; u < 4; ++u) {
                        const uint32_t q = q0 + u * NT, b = bin(kx[u]);
                        if (q < m && b >= r_lo && b <= r_hi) {
                            const uint32_t pos = L.off[padded<P>(b)] - base + atomicAdd(&L.cur[b], 1u);
                            L.kx[pos] = kx[u];
                            L.ky[pos] = w.sky[q];
                            L.row[pos] = w.surv[q];
                            L.bin[pos] = (uint16_t)(b | (w.dead[q] ? kDeadBit : 0));
                        }
                    }
                }
                nf = staged_front(L, cnt, base, r_lo, r_hi, emit);
            } else {
                nf = unstaged_front(L, w, bin, r_lo, r_hi, emit);
            }
            n_front += nf;
            r_lo = r_hi + 1;
        }
    }
    if (t == 0) {
        sc->part_lo[part] = g_lo;
        sc->part_cnt[part] = n_front;
    }
    // The ticket: everything this part wrote is visible to the part that draws the last one.  One thread
    // fences for the block, after every thread's stores have been acknowledged and the block has met (a
    // fence per wave costs a cache write-back each: 1 024 of them took most of the kernel's time).
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (t == 0) {
        __threadfence();
        const bool last = atomicAdd(&sc->counters[1], 1u) == n_parts - 1;
        if (last) __threadfence();
        L.is_last = last ? 1u : 0u;
    }
    __syncthreads();
    if (!L.is_last) return;
    if (t < kWave) {
        const uint32_t c = t < n_parts ? sc->part_cnt[t] : 0u;
        const uint32_t incl = wave_scan_sum(c);
        L.part_base[t] = incl - c;
        L.part_cnt[t] = c;
        L.part_lo[t] = t < n_parts ? sc->part_lo[t] : 0u;
        if (t == kWave - 1) {
            out_count[0] = incl;
            sc->counters[1] = 0;
        }
    }
    __syncthreads();
    for (uint32_t p = 0; p < n_parts; ++p) {
        const uint32_t c = L.part_cnt[p], lo = L.part_lo[p];
        const uint64_t base = L.part_base[p];
        for (uint32_t i0 = t; i0 < c; i0 += 8 * NT) {   // eight loads in flight per thread
            uint32_t v[8];
#pragma unroll
            for (uint32_t u = 0; u < 8; ++u) v[u] = w.staged[lo + (i0 + u * NT < c ? i0 + u * NT : i0)];
#pragma unroll
            for (uint32_t u = 0; u < 8; ++u) {
                const uint32_t i = i0 + u * NT;
                if (i < c && base + i < capacity) out_idx[base + i] = v[u];
            }
        }
    }
}

// Blocks of the launch: 0 finishes the front; 1 runs a waiting top-k merge (only launched with one); the
// others return at once unless more than kStage rows survived, and then share the large front with block 0.
__global__ __launch_bounds__(kFinishThreads) void pareto_finish_kernel(ParetoWs w, uint32_t n, SelectScratch *sc,
                                                                        uint64_t *out_idx,
                                                                        uint64_t capacity, uint64_t *out_count,
                                                                        MergeRider rider) {
    const uint32_t first_helper = rider.n_blocks ? 2 : 1;
    if (rider.n_blocks && blockIdx.x == 1) {
        if (rider.K == 1)
            topk_merge_body<1, kFinishThreads>(rider.w, rider.n_blocks, rider.k, rider.out_idx, rider.out_val, rider.out_cnt);
        else if (rider.K == 2)
            topk_merge_body<2, kFinishThreads>(rider.w, rider.n_blocks, rider.k, rider.out_idx, rider.out_val, rider.out_cnt);
        else if (rider.K == 3)
            topk_merge_body<3, kFinishThreads>(rider.w, rider.n_blocks, rider.k, rider.out_idx, rider.out_val, rider.out_cnt);
        else
            topk_merge_body<4, kFinishThreads>(rider.w, rider.n_blocks, rider.k, rider.out_idx, rider.out_val, rider.out_cnt);
        return;
    }
    static_assert(kFinishThreads == 1024, "kPerFinish assumes 1024 threads");
    constexpr uint32_t P = kPerFinish;
    __shared__ FinishLds L;
    const uint32_t t = threadIdx.x;
    const bool helper = blockIdx.x >= first_helper;     // block-uniform
    if (helper && sc->counters[0] <= kStage) return;
    if (threadIdx.x == 0) L.nfront = 0;
    // Everything the finishing block reads from global memory is requested at once, before the survivor
    // count is known: the first kStage survivor records (index clamped to the workspace's n rows; entries
    // at or beyond the count are ignored later), the count and the sample partials.
    constexpr uint32_t kPer = kStage / kFinishThreads;
    uint64_t rx[kPer], ry[kPer];
    uint32_t rr[kPer];
    if (!helper) {
#pragma unroll
        for (uint32_t q = 0; q < kPer; ++q) {
            const uint32_t j = q * kFinishThreads + t, jc = j < n ? j : n - 1;
            rx[q] = w.skx[jc];
            ry[q] = w.sky[jc];
            rr[q] = w.surv[jc];
        }
    }
    const uint32_t m = sc->counters[0];
    // the tables of the staged path are put into their neutral state while the loads are under way
    for (uint32_t i = t; i < padded_size<P>(); i += kFinishThreads) L.lower[i] = kNone;
#pragma unroll
    for (uint32_t q = 0; q < kPerFinish; ++q) {
        const uint32_t i = q * kFinishThreads + t;
        L.rep[i] = kNone;
        L.cur[i] = 0;
    }
    const Binning bin = sampled_binning(sc, L.rng);     // its barrier also covers the tables above
    if (m > kStage) {
        pareto_large_front(L, w, sc, bin, m, helper ? blockIdx.x - first_helper + 1 : 0, gridDim.x - first_helper + 1,
                           out_idx, capacity, out_count);
        return;
    }
    // Survivors that are dominated for sure are dropped first (after the staircase and survivors kernels there
    // are few; the filter pass leaves more): those with a survivor of a strictly lower bin at or below their y,
    // and those that their own bin's representative dominates -- the survivor with the bin's least y (of those,
    // the least x); rows often tie in x, and then the representative settles all of them but the ties in y.
    // Tables: least y per bin in the LDS that the records are staged in afterwards, then its exclusive
    // prefix-min; the representatives' x in the LDS of the bin counts.
    uint32_t rb[kPer];
    bool live[kPer];
#pragma unroll
    for (uint32_t q = 0; q < kPer; ++q) {
        rb[q] = bin(rx[q]);
        live[q] = q * kFinishThreads + t < m;
        if (live[q]) atomicMin((unsigned long long *)&L.lower[padded<P>(rb[q])], (unsigned long long)ry[q]);
    }
    __syncthreads();
    uint64_t bin_y[kPer];                               // least y of the record's own bin
#pragma unroll
    for (uint32_t q = 0; q < kPer; ++q) {
        bin_y[q] = L.lower[padded<P>(rb[q])];
        if (live[q] && ry[q] == bin_y[q]) atomicMin((unsigned long long *)&L.rep[rb[q]], (unsigned long long)rx[q]);
    }
    __syncthreads();
    scan_min_excl<kFinishThreads>(L.lower, L.tmp64);
    bool alive[kPer];
#pragma unroll
    for (uint32_t q = 0; q < kPer; ++q) {
        const uint64_t rep_x = L.rep[rb[q]];
        const bool by_rep = rep_x <= rx[q] && (rep_x < rx[q] || bin_y[q] < ry[q]);     // bin_y <= ry always
        alive[q] = live[q] && ry[q] < L.lower[padded<P>(rb[q])] && !by_rep;
    }
    __syncthreads();                                    // both tables have been read by everyone
#pragma unroll
    for (uint32_t q = 0; q < kPerFinish; ++q) {
        const uint32_t i = q * kFinishThreads + t;
        L.off[padded<P>(i)] = 0;
        L.foff[padded<P>(i)] = 0;
    }
    if (t == 0) L.off[padded<P>(kBins)] = 0;
    __syncthreads();
#pragma unroll
    for (uint32_t q = 0; q < kPer; ++q)
        if (alive[q]) atomicAdd(&L.off[padded<P>(rb[q])], 1u);
    __syncthreads();                                    // records may be staged from here on
    scan_sum_excl<kFinishThreads, true>(L.off, L.tmp);
    const uint32_t m_alive = L.off[padded<P>(kBins)];
    // records staged in LDS, grouped by bin
#pragma unroll
    for (uint32_t q = 0; q < kPer; ++q) {
        if (alive[q]) {
            const uint32_t pos = L.off[padded<P>(rb[q])] + atomicAdd(&L.cur[rb[q]], 1u);
            L.kx[pos] = rx[q]; L.ky[pos] = ry[q]; L.row[pos] = rr[q]; L.bin[pos] = (uint16_t)rb[q];
        }
    }
    const uint32_t n_front = staged_front(L, m_alive, 0, 0, kBins - 1, [&](uint32_t pos, uint32_t row) {
        if (pos < capacity) out_idx[pos] = row;
    });
    if (t == 0) out_count[0] = n_front;
}

__global__ void pareto_empty_kernel(uint64_t *out_count) { out_count[0] = 0; }

// A row chunk asked for by the caller is taken when batches of 8 or of 6 rows per thread tile it; otherwise the
// passes deal their own batches.  Calls fn(chunk, integral_constant<rows per thread>).
template <typename F>
void with_row_chunk(uint32_t row_chunk, F &&fn) {
    if (row_chunk && row_chunk % (kBlock * 8) == 0) fn(row_chunk, std::integral_constant<uint32_t, 8>{});
    else if (row_chunk && row_chunk % (kBlock * 6) == 0) fn(row_chunk, std::integral_constant<uint32_t, 6>{});
    else fn(kDefaultChunk, std::integral_constant<uint32_t, 8>{});
}

template <int K>
void launch_top1_pass(const guide_select_spec &spec, uint64_t n, void *ws, const SampleRider &sample, hipStream_t stream,
                      uint32_t row_chunk) {
    const uint32_t nb = blocks_for(n);
    with_max_constraints(spec.n_constraints, [&](auto maxc) {
        with_row_chunk(row_chunk, [&](uint32_t chunk, auto u) {
            hipLaunchKernelGGL((topk_pass_kernel<K, decltype(maxc)::value, decltype(u)::value>),
                               dim3(nb + (sample.on ? kSampleBlocks : 0)), dim3(kBlock), 0, stream, spec.objective,
                               make_filter(spec), (uint32_t)n, top1_ws(ws), nb, sample, chunk);
        });
    });
}
// Pairs per block partial for a request of k (the pass kernel's template argument).
int partial_width(uint32_t k) { return k <= 4 ? (int)k : 8; }
void launch_top1_pass(const guide_select_spec &spec, uint64_t n, void *ws, const SampleRider &sample, hipStream_t stream,
                      uint32_t chunk = 0) {
    switch (partial_width(spec.k)) {
        case 1: launch_top1_pass<1>(spec, n, ws, sample, stream, chunk); break;
        case 2: launch_top1_pass<2>(spec, n, ws, sample, stream, chunk); break;
        case 3: launch_top1_pass<3>(spec, n, ws, sample, stream, chunk); break;
        case 4: launch_top1_pass<4>(spec, n, ws, sample, stream, chunk); break;
        default: launch_top1_pass<8>(spec, n, ws, sample, stream, chunk); break;
    }
}
void launch_top1_merge(int K, void *ws, uint32_t n_blocks, uint32_t k, const guide_select_out &out, hipStream_t stream) {
    const Top1Ws w = top1_ws(ws);
    const dim3 one(1), nt(kMergeThreads);
    switch (K) {
        case 1: hipLaunchKernelGGL(topk_merge_kernel<1>, one, nt, 0, stream, w, n_blocks, k, out.idx, out.val, out.count); break;
        case 2: hipLaunchKernelGGL(topk_merge_kernel<2>, one, nt, 0, stream, w, n_blocks, k, out.idx, out.val, out.count); break;
        case 3: hipLaunchKernelGGL(topk_merge_kernel<3>, one, nt, 0, stream, w, n_blocks, k, out.idx, out.val, out.count); break;
        case 4: hipLaunchKernelGGL(topk_merge_kernel<4>, one, nt, 0, stream, w, n_blocks, k, out.idx, out.val, out.count); break;
        default: hipLaunchKernelGGL(topk_merge_kernel<8>, one, nt, 0, stream, w, n_blocks, k, out.idx, out.val, out.count); break;
    }
}

}  // namespace

static_assert(sizeof(SelectScratch) <= kSelectScratchMax, "kSelectScratchMax is too small");
size_t select_scratch_bytes() { return sizeof(SelectScratch); }


size_t select_workspace_bytes(const guide_select_spec &spec, uint64_t n) {
    if (spec.mode == GUIDE_SELECT_PARETO) return pareto_ws_bytes(n);
    const size_t a = topk_ws_bytes(spec.n_groups ? spec.n_groups : 1), b = top1_ws_bytes();
    return a > b ? a : b;
}

hipError_t launch_select_topk(const guide_select_spec &spec, uint64_t n, const guide_select_out &out, void *ws,
                              void *scratch, hipStream_t stream) {
    (void)scratch;
    if (!spec.group) {
        launch_top1_pass(spec, n, ws, SampleRider{}, stream);
        launch_top1_merge(partial_width(spec.k), ws, blocks_for(n), spec.k, out, stream);
        return hipGetLastError();
    }
    const uint32_t G = spec.n_groups;
    const TopkWs w = topk_ws(ws, G);
    const RowFilter f = make_filter(spec);
    const uint32_t nb = blocks_for(n);
    for (uint32_t round = 0; round < spec.k; ++round) {
        hipLaunchKernelGGL(topk_round_kernel, dim3(nb), dim3(kBlock), 0, stream, spec.objective, f, spec.group, G,
                           (uint32_t)n, round, w);
        hipLaunchKernelGGL(topk_final_kernel, dim3(G), dim3(kBlock), 0, stream, w, G, nb, round, spec.k, out.idx, out.val,
                           out.count);
    }
    return hipGetLastError();
}

// A launch with the timing events attached to its dispatch when there are any.
template <typename Kernel, typename... Args>
static void launch_timed(Kernel kernel, dim3 grid, dim3 block, hipStream_t stream, const LaunchTiming *tm, Args... args) {
    if (tm && tm->start) hipExtLaunchKernelGGL(kernel, grid, block, 0, stream, tm->start, tm->stop, 0, args...);
    else hipLaunchKernelGGL(kernel, grid, block, 0, stream, args...);
}

// The passes after the row sample: the filter pass (with the per-lane lists of a top-k that shares the
// columns) and the finishing kernel.  tm: two event pairs (filter, finish) or none.
static hipError_t launch_pareto_passes(const guide_select_spec &spec, uint64_t n, const guide_select_out &out, void *ws,
                                       SelectScratch *sc, const MergeRider &rider, hipStream_t stream,
                                       const SharedTopk *shared = nullptr, int shared_k = 0, uint32_t row_chunk = 0,
                                       const LaunchTiming *tm = nullptr) {
    const LaunchTiming *tm_filter = tm, *tm_fin = tm ? tm + 1 : nullptr;
    const ParetoWs w = pareto_ws(ws, n);
    const RowFilter f = make_filter(spec);
    const uint32_t nb = pareto_blocks(n), n32 = (uint32_t)n;
    const double *x = spec.objective, *y = spec.objective_y;
    const dim3 grid(nb), block(kBlock);
    with_row_chunk(row_chunk, [&](uint32_t chunk, auto u) {
        constexpr uint32_t U = decltype(u)::value;
        if (shared) {       // only offered for a Pareto selection without constraint columns
            const SharedTopk t = *shared;
            if (shared_k == 1) launch_timed(pareto_filter_kernel<0, 1, U>, grid, block, stream, tm_filter, x, y, f, n32, w, sc, t, chunk);
            else if (shared_k == 2) launch_timed(pareto_filter_kernel<0, 2, U>, grid, block, stream, tm_filter, x, y, f, n32, w, sc, t, chunk);
            else if (shared_k == 3) launch_timed(pareto_filter_kernel<0, 3, U>, grid, block, stream, tm_filter, x, y, f, n32, w, sc, t, chunk);
            else launch_timed(pareto_filter_kernel<0, 4, U>, grid, block, stream, tm_filter, x, y, f, n32, w, sc, t, chunk);
            return;
        }
        with_max_constraints(f.n_con, [&](auto maxc) {
            constexpr uint32_t MAXC = decltype(maxc)::value;
            launch_timed(pareto_filter_kernel<MAXC, 0, U>, grid, block, stream, tm_filter, x, y, f, n32, w, sc, SharedTopk{},
                         chunk);
        });
    });
    const uint32_t helpers = n > kStage ? kLargeParts - 1 : 0;     // no more than kStage rows: the staged path for sure
    launch_timed(pareto_finish_kernel, dim3((rider.n_blocks ? 2 : 1) + helpers), dim3(kFinishThreads), stream, tm_fin, w, n32,
                 sc, out.idx, out.capacity, out.count, rider);
    return hipGetLastError();
}

hipError_t launch_select_pareto(const guide_select_spec &spec, uint64_t n, const guide_select_out &out, void *ws,
                                void *scratch, hipStream_t stream) {
    if (n == 0) {
        hipLaunchKernelGGL(pareto_empty_kernel, dim3(1), dim3(1), 0, stream, out.count);
        return hipGetLastError();
    }
    SelectScratch *sc = (SelectScratch *)scratch;
    hipLaunchKernelGGL(pareto_prepare_kernel, dim3(kSampleBlocks), dim3(kBlock), 0, stream, spec.objective,
                       spec.objective_y, make_filter(spec), (uint32_t)n, sc);
    return launch_pareto_passes(spec, n, out, ws, sc, MergeRider{}, stream);
}

// True when the top-k selection reads only the Pareto selection's x, y and flag columns (and the Pareto
// selection has no constraint columns); fills the description for the staircase kernel.
static bool shares_columns(const guide_select_spec &topk, const guide_select_spec &pareto, SharedTopk *t) {
    const double *x = pareto.objective, *y = pareto.objective_y;
    if (pareto.n_constraints != 0 || topk.n_constraints > 2 || topk.k > 4) return false;
    if (topk.objective != x && topk.objective != y) return false;
    if (topk.feasible && topk.feasible != pareto.feasible) return false;
    memset(t, 0, sizeof *t);
    t->obj_is_y = topk.objective == y ? 1u : 0u;
    t->use_feasible = topk.feasible ? 1u : 0u;
    t->n_con = topk.n_constraints;
    for (uint32_t c = 0; c < topk.n_constraints; ++c) {
        const double *col = topk.constraints[c].column;
        if (col != x && col != y) return false;
        t->con_is_y[c] = col == y ? 1u : 0u;
        t->cap[c] = topk.constraints[c].cap;
    }
    return true;
}

// A top-k selection (one group) and a Pareto selection over the same n > 0 rows in three launches
// instead of five.  The top-k merge rides along with the finishing kernel of the Pareto front (for block
// partials of up to 4 pairs; wider ones merge alone).  When the top-k reads only the Pareto selection's
// columns, its pass is folded into the filter pass (sample, filter + lists, finish + merge); otherwise the
// Pareto row sample rides along with the top-k pass (pass + sample, filter, finish + merge).
// sampled: the caller's own kernel has taken the row sample.
hipError_t launch_select_both(const guide_select_spec &topk, const guide_select_out &topk_out, void *topk_ws,
                              const guide_select_spec &pareto, const guide_select_out &pareto_out, void *pareto_ws_,
                              uint64_t n, void *scratch, hipStream_t stream, bool sampled,
                              uint32_t row_chunk, const LaunchTiming *pass_timing) {
    SelectScratch *sc = (SelectScratch *)scratch;
    const int K = partial_width(topk.k);
    SharedTopk shared;
    const bool folded = shares_columns(topk, pareto, &shared);
    if (folded) {
        shared.w = top1_ws(topk_ws);
        if (!sampled)
            hipLaunchKernelGGL(pareto_prepare_kernel, dim3(kSampleBlocks), dim3(kBlock), 0, stream, pareto.objective,
                               pareto.objective_y, make_filter(pareto), (uint32_t)n, sc);
    } else {
        const SampleRider sample{sampled ? 0u : 1u, pareto.objective, pareto.objective_y, make_filter(pareto), sc};
        launch_top1_pass(topk, n, topk_ws, sample, stream, row_chunk);
    }
    MergeRider rider{};
    if (K <= 4)
        rider = MergeRider{top1_ws(topk_ws), folded ? pareto_blocks(n) : blocks_for(n), topk.k, (uint32_t)K, topk_out.idx,
                           topk_out.val, topk_out.count};       // partials: one per block of the kernel that kept the lists
    else
        launch_top1_merge(K, topk_ws, blocks_for(n), topk.k, topk_out, stream);
    return launch_pareto_passes(pareto, n, pareto_out, pareto_ws_, sc, rider, stream, folded ? &shared : nullptr, K, row_chunk,
                                pass_timing);
}

// The passes after the sample, for a caller whose own kernel has taken the row sample.
// merge_ws != nullptr: the merge of a folded top-k (merge_blocks block partials of kFusedTopK pairs) rides
// along with the finishing kernel instead of taking a launch of its own.
hipError_t launch_pareto_sampled(const guide_select_spec &spec, uint64_t n, const guide_select_out &out, void *ws,
                                 void *scratch, void *merge_ws, uint32_t merge_blocks,
                                 uint32_t merge_k, const guide_select_out *merge_out, hipStream_t stream,
                                 uint32_t row_chunk) {
    MergeRider rider{};
    if (merge_ws)
        rider = MergeRider{top1_ws(merge_ws), merge_blocks, merge_k, (uint32_t)kFusedTopK, merge_out->idx, merge_out->val,
                           merge_out->count};
    return launch_pareto_passes(spec, n, out, ws, (SelectScratch *)scratch, rider, stream, nullptr, 0, row_chunk);
}

size_t topk_partials_bytes() { return top1_ws_bytes(); }

// Merge of n_blocks block partials of kFusedTopK pairs each.
hipError_t launch_topk_merge(void *ws, uint32_t n_blocks, uint32_t k, const guide_select_out &out, hipStream_t stream) {
    launch_top1_merge(kFusedTopK, ws, n_blocks, k, out, stream);
    return hipGetLastError();
}

}  // namespace guide
