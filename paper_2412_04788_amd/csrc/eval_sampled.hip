// Random-sampled configuration space: candidate i is drawn from a counter-based
// generator keyed by (seed, i), evaluated, and folded into reduced outputs
// (feasible count, per model-size bucket best candidate, latency histogram)
// inside the kernel.  Only a few KB leave the chip.
#include "kernels.hpp"
#include "perf_model.hpp"
#include "reduce.hpp"

namespace guide {

namespace {

constexpr uint32_t kMaxBuckets = GUIDE_MAX_BUCKET_EDGES + 1;

// Philox4x64-10 (Salmon, Moraes, Dror, Shaw, SC'11): ten rounds, each two
// 64x64 -> 128 bit multiplies by the published constants; the key advances by
// the Weyl increments between rounds.
struct Block256 {
    uint64_t v[4];
};
__device__ inline Block256 philox4x64_10(uint64_t c0, uint64_t c1, uint64_t c2, uint64_t c3, uint64_t k0, uint64_t k1) {
    constexpr uint64_t M0 = 0xD2E7470EE14C6C93ull, M1 = 0xCA5A826395121157ull;
    constexpr uint64_t W0 = 0x9E3779B97F4A7C15ull, W1 = 0xBB67AE8584CAA73Bull;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t hi0 = __umul64hi(M0, c0), lo0 = M0 * c0;
        const uint64_t hi1 = __umul64hi(M1, c2), lo1 = M1 * c2;
        const uint64_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += W0; k1 += W1;
    }
    Block256 b;
    b.v[0] = c0; b.v[1] = c1; b.v[2] = c2; b.v[3] = c3;
    return b;
}

struct SampledLds {
    uint32_t heads[GUIDE_LATTICE], batch[GUIDE_LATTICE], s_in[GUIDE_LATTICE], s_out[GUIDE_LATTICE];
    double r_peak[GUIDE_LATTICE], r_bw[GUIDE_LATTICE];
    uint64_t win_key[kBlock / kWave][kMaxBuckets], win_idx[kBlock / kWave][kMaxBuckets];
    uint32_t hist[GUIDE_HIST_BINS];
    uint32_t feasible[kBlock / kWave];
};

// Block partials of the bucket winners: [block][bucket] keys, then rows.
struct SampledScratch {
    uint64_t key[kSampledMaxBlocks][kMaxBuckets];
    uint64_t idx[kSampledMaxBlocks][kMaxBuckets];
};

__global__ void sampled_init_kernel(guide_sampled_out out) {
    const uint32_t i = threadIdx.x;
    if (i < GUIDE_HIST_BINS) out.hist[i] = 0;
    if (i == 0) out.feasible_count[0] = 0;
}

// 16-bit field j of the block (lowest field of word 0 first).
__device__ inline uint32_t field(const Block256 &b, int j) { return (uint32_t)(b.v[j >> 2] >> (16 * (j & 3))) & 0xFFFFu; }

template <bool ADDITIVE>
__global__ __launch_bounds__(kBlock) void eval_sampled_kernel(const SpaceTables *__restrict__ tab, uint64_t seed,
                                                              uint64_t first, uint64_t count, double ttft_cap,
                                                              guide_sampled_out out, SampledScratch *scratch) {
    __shared__ SampledLds s;
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    for (uint32_t i = threadIdx.x; i < GUIDE_LATTICE; i += kBlock) {
        s.heads[i] = tab->heads[i];
        s.batch[i] = tab->batch[i];
        s.s_in[i] = tab->s_in[i];
        s.s_out[i] = tab->s_out[i];
        s.r_peak[i] = 1.0 / tab->peak[i];
        s.r_bw[i] = 1.0 / tab->bw[i];
    }
    for (uint32_t i = threadIdx.x; i < (kBlock / kWave) * kMaxBuckets; i += kBlock) {
        (&s.win_key[0][0])[i] = kNone;
        (&s.win_idx[0][0])[i] = kNone;
    }
    for (uint32_t i = threadIdx.x; i < GUIDE_HIST_BINS; i += kBlock) s.hist[i] = 0;
    __syncthreads();
    const uint32_t n_edges = tab->n_edges;
    const double link_div = tab->link_div;
    uint32_t n_feasible = 0;
    const uint64_t stride = (uint64_t)gridDim.x * kBlock;
    const uint64_t iters = (count + stride - 1) / stride;   // same trip count for every lane
    for (uint64_t it = 0; it < iters; ++it) {
        const uint64_t i = it * stride + (uint64_t)blockIdx.x * kBlock + threadIdx.x;
        const bool live = i < count;
        bool feasible = false, wins = false;
        Pair cand = {kNone, kNone};
        uint32_t bucket = 0;
        if (live) {
            const uint64_t id = first + i;
            const Block256 r = philox4x64_10(id, 0, 0, 0, seed, 0);
            guide_model md;
            md.L = tab->layers_lo + ((field(r, 0) * tab->layers_n) >> 16);
            md.n_h = s.heads[field(r, 1) >> 6];
            md.d = 128u * md.n_h;
            const uint32_t kvc = tab->kv_choices[field(r, 2) >> 14];
            md.n_kv = kvc ? kvc : md.n_h;
            // d_ff = 128 * floor(ratio * n_h + 1/2), ratio = (lo_x2 + span_x2 * u / 65536) / 2
            const uint64_t num = ((uint64_t)tab->ffn_lo_x2 * 65536u + (uint64_t)tab->ffn_span_x2 * field(r, 3)) * md.n_h + 65536u;
            md.d_ff = 128u * (uint32_t)(num >> 17);
            md.V = tab->vocab;
            md.E = 1;
            md.k = 1;
            Knobs kn;
            kn.b = s.batch[field(r, 7) >> 6];
            kn.s_in = s.s_in[field(r, 8) >> 6];
            kn.s_out = s.s_out[field(r, 9) >> 6];
            kn.p = tab->tp[field(r, 10) >> 14];
            kn.wbits = tab->wbits[(field(r, 11) * 3u) >> 16];
            kn.blk = tab->kv_block[field(r, 12) >> 15];
            kn.mbt = tab->mbt[(field(r, 13) * 3u) >> 16];
            const double r_peak = s.r_peak[field(r, 4) >> 6], r_bw = s.r_bw[field(r, 5) >> 6];
            const double cap = tab->cap[(field(r, 6) * 6u) >> 16];

            const Coef cf = make_coef(md, kn.p, kn.wbits);
            const TimeCoef tc = make_time_coef(cf, r_peak, r_bw, link_div * r_bw, 0.0);
            EvalResult ev;
            ev.t_prefill = prefill_time_fast<ADDITIVE>(tc, kn.b, kn.s_in, kn.mbt, recip_up(fast_recip((double)kn.s_in)),
                                                       recip_up(fast_recip((double)kn.mbt)));
            ev.t_decode = decode_time_fast<ADDITIVE>(tc, kn.b, kn.s_in, kn.s_out - 1);
            const MemResult mem = memory_check(cf, cap, kn.b, kn.s_in, kn.s_out, kn.blk);
            const double t_batch = ev.t_prefill + ev.t_decode;
            const double cost = (double)kn.p * (1.0e6 / 3600.0) * t_batch * fast_recip((double)kn.b * (double)kn.s_out);
            for (uint32_t e = 0; e < n_edges; ++e) bucket += cf.p_total >= tab->edges[e] ? 1u : 0u;
            feasible = mem.feasible;
            if (feasible) {
                ++n_feasible;
                // 8 bins per octave from the exponent and the top three mantissa bits
                long long bin = (long long)((uint64_t)__double_as_longlong(t_batch) >> 49) - (long long)((1023 - 12) << 3);
                bin = bin < 0 ? 0 : (bin > GUIDE_HIST_BINS - 1 ? GUIDE_HIST_BINS - 1 : bin);
                atomicAdd(&s.hist[bin], 1u);
                wins = ev.t_prefill <= ttft_cap && cost == cost;
                cand.key = key_of(cost);
                cand.idx = id;
            }
            if (out.t_prefill) out.t_prefill[i] = ev.t_prefill;
            if (out.t_batch) out.t_batch[i] = t_batch;
            if (out.cost) out.cost[i] = cost;
            if (out.b_max) out.b_max[i] = mem.b_max;
            if (out.feasible) out.feasible[i] = feasible ? 1 : 0;
            if (out.bucket) out.bucket[i] = bucket;
        }
        slot_update(s.win_key[wave], s.win_idx[wave], bucket, wins, cand);
    }
    for (int off = kWave / 2; off > 0; off >>= 1) n_feasible += __shfl_xor(n_feasible, off, kWave);
    if (lane == 0) s.feasible[wave] = n_feasible;
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < GUIDE_HIST_BINS; i += kBlock)
        if (s.hist[i]) atomicAdd((unsigned long long *)&out.hist[i], (unsigned long long)s.hist[i]);
    if (threadIdx.x == 0) {
        unsigned long long f = 0;
        for (int wv = 0; wv < kBlock / kWave; ++wv) f += s.feasible[wv];
        if (f) atomicAdd((unsigned long long *)out.feasible_count, f);
    }
    for (uint32_t b = threadIdx.x; b <= n_edges; b += kBlock) {
        Pair best = {s.win_key[0][b], s.win_idx[0][b]};
        for (int wv = 1; wv < kBlock / kWave; ++wv) {
            const Pair o = {s.win_key[wv][b], s.win_idx[wv][b]};
            best = pair_min(best, o);
        }
        scratch->key[blockIdx.x][b] = best.key;
        scratch->idx[blockIdx.x][b] = best.idx;
    }
}

// One wave per bucket: least (cost, index) over the block partials.
__global__ __launch_bounds__(kWave) void sampled_final_kernel(const SampledScratch *__restrict__ scratch,
                                                              uint32_t n_blocks, guide_sampled_out out) {
    const uint32_t b = blockIdx.x;
    Pair best = {kNone, kNone};
    for (uint32_t i = threadIdx.x; i < n_blocks; i += kWave) {
        const Pair o = {scratch->key[i][b], scratch->idx[i][b]};
        best = pair_min(best, o);
    }
    best = wave_min(best);
    if (threadIdx.x == 0) {
        out.win_idx[b] = best.idx;
        out.win_val[b] = best.idx == kNone ? INFINITY : value_of(best.key);
    }
}

}  // namespace

size_t sampled_scratch_bytes() { return sizeof(SampledScratch); }

hipError_t launch_eval_sampled(const SpaceTables *tab, uint64_t seed, uint64_t first, uint64_t count, double ttft_cap,
                               bool additive, const guide_sampled_out &out, void *scratch, hipStream_t stream,
                               uint32_t n_edges) {
    uint64_t need = (count + kBlock - 1) / kBlock;
    if (need == 0) need = 1;
    const uint32_t nb = (uint32_t)(need < kSampledMaxBlocks ? need : kSampledMaxBlocks);
    SampledScratch *sc = (SampledScratch *)scratch;
    hipLaunchKernelGGL(sampled_init_kernel, dim3(1), dim3(GUIDE_HIST_BINS), 0, stream, out);
    if (additive)
        hipLaunchKernelGGL(eval_sampled_kernel<true>, dim3(nb), dim3(kBlock), 0, stream, tab, seed, first, count,
                           ttft_cap, out, sc);
    else
        hipLaunchKernelGGL(eval_sampled_kernel<false>, dim3(nb), dim3(kBlock), 0, stream, tab, seed, first, count,
                           ttft_cap, out, sc);
    hipLaunchKernelGGL(sampled_final_kernel, dim3(n_edges + 1), dim3(kWave), 0, stream, (const SampledScratch *)sc, nb,
                       out);
    return hipGetLastError();
}

}  // namespace guide
