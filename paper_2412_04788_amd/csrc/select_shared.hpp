// Pieces of the selection kernels that the grid evaluation also uses when
// selections are folded into it: per-lane top-K lists and their block merge,
// the layout of the top-k block partials, and the scratch of the Pareto kernels.
#pragma once

#include "reduce.hpp"

namespace guide {

constexpr uint32_t kSelBlocks = 1024;      // most blocks of a streaming pass (four per CU)

// Context-owned device scratch of the Pareto kernels.  The kernel of a call that takes
// the row sample puts what the later ones accumulate into (the survivor counter, the
// ticket counter) into its neutral state, so the scratch needs no set-up and no call
// depends on how the previous one ended.
constexpr uint32_t kBins = 4096;
constexpr uint32_t kSampleBlocks = 64;           // blocks of kBlock rows each that take the row sample (a kernel of their own or riders)
constexpr uint32_t kSampleFrontPer = 32;         // sample rows that one such block hands to the filter pass, at most
struct SelectScratch {
    uint32_t counters[4];          // [0] survivors appended, [1] tickets drawn by the parts of a large front
    uint64_t sample_lo[kSampleBlocks];       // per sampling block: least x key of passing sample rows
    Pair sample_best[kSampleBlocks];         // per sampling block: (least y key, its x key)
    uint32_t part_lo[64], part_cnt[64];   // large-front path only: per part, its first survivor slot and its front members
    Pair sample_front[kSampleBlocks * kSampleFrontPer];   // (y key, x key) of sample rows that prune; unused slots kNone
};

// Sample number -> row for blocks that take a sample of their own: block rb's kBlock samples are spread over
// the whole range (sample k = thread * n_blocks + rb), and a sample sits at a scrambled place inside its
// stride, so that no period of the rows' layout lines up with the sample.
__device__ inline uint32_t sample_number(uint32_t rb, uint32_t n_blocks) { return threadIdx.x * n_blocks + rb; }
__device__ inline uint32_t sample_row(uint32_t k, uint32_t stride) {
    return k * stride + ((k * 2654435761u) >> 8) % stride;
}

// The rows of a sampling block's sample that are worth handing to the filter pass of a Pareto selection: a
// sample row prunes every row with a larger x (in a higher bin) and y not below its own, so a sample row with
// another one at or below it in both x and y adds nothing.  Every thread of the block brings one sample row
// (pass = false: none).  Each wave hands over the front of its rows from the right: the row with the least y
// (of those, the least x), then the row with the least y among the rows left of it, and so on, at most
// kSampleFrontPer / waves of them (the rows further left prune the least; any subset is valid).  The wave's
// unused slots are filled with kNone.
__device__ inline void store_sample_front(bool pass, uint64_t kx, uint64_t ky, Pair *slots) {
    constexpr uint32_t kPerWave = kSampleFrontPer / (kBlock / kWave);
    const uint32_t lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    uint64_t bound = kNone;                             // rows at or right of this x are done with
    Pair mine = {kNone, kNone};
    for (uint32_t it = 0; it < kPerWave; ++it) {        // wave-uniform trip count
        const bool in = pass && kx < bound;
        const Pair p = wave_min(in ? Pair{ky, kx} : Pair{kNone, kNone});
        if (p.idx == kNone) break;                      // no row left (x keys of rows are below kNone)
        if (lane == it) mine = p;
        bound = p.idx;
    }
    if (lane < kPerWave) slots[wave * kPerWave + lane] = mine;
}

// Sorted list of the K least (key, row) pairs seen by one lane.
template <int K>
struct TopList {
    Pair v[K];
    __device__ void init() {
#pragma unroll
        for (int i = 0; i < K; ++i) v[i] = Pair{kNone, kNone};
    }
    __device__ void insert(const Pair &p) {
        if (!less_than(p, v[K - 1])) return;
        v[K - 1] = p;
#pragma unroll
        for (int i = K - 1; i > 0; --i) {
            if (less_than(v[i], v[i - 1])) {
                const Pair t = v[i];
                v[i] = v[i - 1];
                v[i - 1] = t;
            }
        }
    }
    // insert() for a caller whose rows arrive in ascending order: the new row is larger than every row
    // in the list, so it goes before exactly the entries with a larger key.  No branches inside: every
    // position takes its left neighbour, the new pair or itself.
    __device__ void insert_ascending(const Pair &p) {
        if (p.key < v[K - 1].key) {
#pragma unroll
            for (int i = K - 1; i > 0; --i) {
                const bool shift = p.key < v[i - 1].key;    // the neighbour moves up into position i
                const bool here = p.key < v[i].key;         // (and not shift:) the new pair lands at i
                v[i].key = shift ? v[i - 1].key : (here ? p.key : v[i].key);
                v[i].idx = shift ? v[i - 1].idx : (here ? p.idx : v[i].idx);
            }
            const bool first = p.key < v[0].key;
            v[0].key = first ? p.key : v[0].key;
            v[0].idx = first ? p.idx : v[0].idx;
        }
    }
    __device__ void pop() {
#pragma unroll
        for (int i = 0; i + 1 < K; ++i) v[i] = v[i + 1];
        v[K - 1] = Pair{kNone, kNone};
    }
};

// The K least pairs over all lanes of the block, in order: emit(r, pair) is called once for every
// r < K by some lane of wave 0 (an empty pair when fewer than r + 1 exist).  NW = waves of the block.
// Stage 1, per wave: K rounds of a key-only minimum; the owner is found by ballot, and only tied
// keys need a second reduction over rows (row numbers fit 32 bits).  Rows are unique, so one lane pops per round.
// Stage 2, wave 0: each of the NW * K candidates counts the candidates before it (lane index
// breaks the tie between empty ones) -- its rank is its output slot.
template <int K, int NW, typename Emit>
__device__ inline void block_topk(TopList<K> &l, Pair (*s_pairs)[K], Emit &&emit) {
    static_assert(NW * K <= kWave, "stage 2 holds one candidate per lane of a wave");
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
#pragma unroll
    for (int r = 0; r < K; ++r) {
        const uint64_t mk = wave_min(l.v[0].key);
        const bool mine = l.v[0].key == mk && l.v[0].idx != kNone;
        const uint64_t tied = __ballot(mine);
        uint64_t mi = kNone;
        if (__popcll(tied) == 1)
            mi = __shfl(l.v[0].idx, __ffsll((long long)tied) - 1, kWave);
        else if (tied)                                  // rows are below 2^32: a 32-bit minimum decides
            mi = wave_min(mine ? (uint32_t)l.v[0].idx : 0xFFFFFFFFu);
        if (mine && l.v[0].idx == mi) l.pop();
        if (lane == 0) s_pairs[wave][r] = Pair{mi == kNone ? kNone : mk, mi};
    }
    __syncthreads();
    if (wave == 0) {
        const Pair *flat = &s_pairs[0][0];
        const Pair c = lane < NW * K ? flat[lane] : Pair{kNone, kNone};
        int rank = 0;
#pragma unroll
        for (int j = 0; j < NW * K; ++j) {
            const Pair o = flat[j];
            rank += (less_than(o, c) || (o.key == c.key && o.idx == c.idx && j < lane)) ? 1 : 0;
        }
        if (lane < NW * K && rank < K) emit(rank, c);
    }
}

// The same result when the caller knows a wave-uniform `bound` with at least K of the wave's
// entries at or below it (or kNone): only entries up to the bound can be among the block's K
// least, and they are few.  Each wave appends them to its LDS segment (a prefix of every lane's
// sorted list; positions from a wave scan of the counts), then wave 0 ranks all of them at once.
// A wave with more than CAP such entries sends the whole block through block_topk instead.
// s_cand: NW x CAP pairs, s_n: NW counters.
template <int K, int NW, int CAP, typename Emit>
__device__ inline void block_topk_bounded(TopList<K> &l, uint64_t bound, Pair (*s_cand)[CAP], uint32_t *s_n,
                                          Pair (*s_pairs)[K], Emit &&emit) {
    static_assert(NW * CAP <= kWave && K <= CAP, "stage 2 holds one candidate per lane of a wave");
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    uint32_t c = 0;
#pragma unroll
    for (int i = 0; i < K; ++i) c += (l.v[i].idx != kNone && l.v[i].key <= bound) ? 1u : 0u;
    const uint32_t incl = wave_scan_sum(c);
    const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, kWave - 1);
    if (total <= (uint32_t)CAP) {
        const uint32_t off = incl - c;
#pragma unroll
        for (int i = 0; i < K; ++i)
            if ((uint32_t)i < c) s_cand[wave][off + i] = l.v[i];
        if (lane < CAP && (uint32_t)lane >= total) s_cand[wave][lane] = Pair{kNone, kNone};
    }
    if (lane == 0) s_n[wave] = total;
    __syncthreads();
    bool overflow = false;
    uint32_t n_valid = 0;
#pragma unroll
    for (int wv = 0; wv < NW; ++wv) {
        overflow = overflow || s_n[wv] > (uint32_t)CAP;
        n_valid += s_n[wv];
    }
    if (overflow) {                                     // block-uniform
        block_topk<K, NW>(l, s_pairs, emit);
        return;
    }
    if (wave == 0) {
        const Pair *flat = &s_cand[0][0];
        const Pair me = lane < NW * CAP ? flat[lane] : Pair{kNone, kNone};
        int rank = 0;
#pragma unroll
        for (int j = 0; j < NW * CAP; ++j) rank += less_than(flat[j], me) ? 1 : 0;
        if (me.idx != kNone && rank < K) emit(rank, me);
        if (lane < K && (uint32_t)lane >= n_valid) emit(lane, Pair{kNone, kNone});
    }
}

// Workspace: part_key[B*K], part_idx[B*K], part_cnt[B].
struct Top1Ws {
    uint64_t *key, *idx, *cnt;
};
__host__ __device__ inline Top1Ws top1_ws(void *ws) {
    Top1Ws w;
    w.key = (uint64_t *)ws;
    w.idx = w.key + (size_t)kSelBlocks * GUIDE_MAX_TOPK;
    w.cnt = w.idx + (size_t)kSelBlocks * GUIDE_MAX_TOPK;
    return w;
}
inline size_t top1_ws_bytes() { return sizeof(uint64_t) * ((size_t)kSelBlocks * (2 * GUIDE_MAX_TOPK + 1)); }

}  // namespace guide
