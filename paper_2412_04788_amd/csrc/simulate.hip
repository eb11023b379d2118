// Step-level continuous-batching simulation, one serving configuration per
// lane, and the per-configuration TTFT percentiles.
//
// The paper states that the frameworks' dynamic batching and split flow are
// simulated (Overview) without giving the procedure; the scheduler simulated
// here is documented in guide.h.  The engine state is kept in aggregated form:
//   - admission is FCFS, so admitted requests are the index range [.., next);
//   - prompt chunks are handed out in admission order, so at most the head of
//     the prefill queue [pf_head, next) is partially prefilled;
//   - a request that finished its prompt decodes on every later step, so its
//     finishing step is known when its prompt completes: decoders live in a
//     per-lane 4-ary min-heap keyed by finishing step (root in registers, the
//     rest in global memory, one cache line per node's children), and their
//     number and total context are two running integers.
// One step therefore costs one pass-time evaluation plus O(1) integer updates;
// heap traffic is O(log n) per request, not per step.
#include <type_traits>

#include "kernels.hpp"
#include "perf_model.hpp"

namespace guide {

namespace {

constexpr uint32_t kSimBlock = 256;      // one block per compute unit: the trace is staged once, the rest of LDS holds heaps
constexpr uint32_t kPctBlock = 256;
constexpr size_t kSimStaticLds = 2 * kSimBlock * 4 + 64;   // the simulation kernel's own static LDS (segment tables)

struct SimLds {
    uint32_t axis[kNumAxes][GUIDE_MAX_AXIS_VALUES];
    guide_model models[GUIDE_MAX_MODELS];
    double arrival[GUIDE_MAX_REQUESTS];
    uint32_t n_in[GUIDE_MAX_REQUESTS];
    uint32_t n_out[GUIDE_MAX_REQUESTS];
};

constexpr uint32_t kKeyBins = 1024;      // buckets of the expected-step-count ordering

// Workspace: heap[position][node] (u64 keys), first[cfg][req] and fin[cfg][req] (time of the first and of the
// last token), then the launch order: perm[position] = configuration, bucket of each configuration, bucket counters.
struct SimWs {
    uint64_t *heap;
    double *first, *fin;
    uint32_t *perm;
    uint32_t *bucket;     // [n_cfg]: bucket of each configuration
    uint32_t *bins;       // [kKeyBins]: counts, then scatter cursors
};
SimWs sim_ws(void *ws, uint32_t n_cfg, uint32_t n_req) {
    SimWs w;
    w.heap = (uint64_t *)ws;
    w.first = (double *)(w.heap + (size_t)n_cfg * n_req);
    w.fin = w.first + (size_t)n_cfg * n_req;
    w.perm = (uint32_t *)(w.fin + (size_t)n_cfg * n_req);
    w.bucket = w.perm + n_cfg;
    w.bins = w.bucket + n_cfg;
    return w;
}

// Grid index -> axis values (s_in / s_out digits are decoded but unused by the simulator).
__device__ inline bool decode_sim_index(const uint32_t (*axis)[GUIDE_MAX_AXIS_VALUES], const GridDesc &g, uint32_t idx,
                                        uint32_t *v) {
    uint32_t rem = idx;
#pragma unroll
    for (int a = kNumAxes - 1; a > 0; --a) {
        const uint32_t q = div32(rem, g.div[a]);
        v[a] = axis[a][rem - q * g.div[a].d];
        rem = q;
    }
    const bool bad = rem >= g.div[0].d;
    v[0] = axis[0][bad ? 0 : rem];
    return bad;
}

// Lanes of a wave run until their slowest configuration ends, so configurations
// are launched in order of a rough estimate of their engine steps: generated
// tokens / concurrency, with concurrency from Little's law (arrival rate x
// latency of a lone request), clamped to [1, sequence cap].  Only the order
// depends on it, never a result.
template <bool ADDITIVE>
__global__ __launch_bounds__(kBlock) void sim_order_count_kernel(GridDesc g, const DevTables *__restrict__ tab,
                                                                 uint32_t n_req,
                                                                 const uint32_t *__restrict__ cfg_idx,
                                                                 const double *__restrict__ rate_in, uint32_t n_cfg,
                                                                 SimWs ws, double sum_in, double sum_out) {
    const double s_sum[2] = {sum_in, sum_out};      // prompt / generated tokens of the whole trace
    const uint32_t c = blockIdx.x * kBlock + threadIdx.x;
    if (c >= n_cfg) return;
    uint32_t v[kNumAxes];
    const bool bad = decode_sim_index(tab->axis_vals, g, cfg_idx[c], v);
    uint32_t b = 0;
    const double rate = rate_in[c];
    if (!bad && rate > 0.0) {
        const guide_hw hw = tab->hw[v[AX_HW]];
        const Coef cf = make_coef(tab->models[v[AX_MODEL]], v[AX_TP], v[AX_WBITS]);
        const TimeCoef tc = make_time_coef(cf, 1.0 / hw.peak_flops, 1.0 / hw.hbm_bw, 1.0 / hw.link_bw, hw.link_lat);
        const double mean_in = s_sum[0] / (double)n_req, mean_out = s_sum[1] / (double)n_req;
        const double ctx = mean_in + 0.5 * mean_out;
        const double lone = mean_out * pass_time<ADDITIVE>(tc, 1.0, ctx, ctx, 1.0) +
                            pass_time<ADDITIVE>(tc, mean_in, mean_in * mean_in, mean_in, 1.0);
        const double conc = fmin(fmax(rate * lone, 1.0), (double)v[AX_BATCH]);
        const float steps = (float)(s_sum[1] / conc);
        const int k = (int)((__log2f(fmaxf(steps, 1.0f)) - 6.0f) * 64.0f);
        b = (uint32_t)(k < 0 ? 0 : (k > (int)kKeyBins - 1 ? (int)kKeyBins - 1 : k));
    }
    ws.bucket[c] = b;
    atomicAdd(&ws.bins[b], 1u);
}

__global__ __launch_bounds__(kKeyBins) void sim_order_scan_kernel(SimWs ws) {
    __shared__ uint32_t s[kKeyBins];
    const uint32_t t = threadIdx.x;
    s[t] = ws.bins[t];
    __syncthreads();
    for (uint32_t off = 1; off < kKeyBins; off <<= 1) {
        const uint32_t o = t >= off ? s[t - off] : 0;
        __syncthreads();
        s[t] += o;
        __syncthreads();
    }
    // longest first: bucket b starts after all higher buckets
    ws.bins[t] = s[kKeyBins - 1] - s[t];
}

__global__ __launch_bounds__(kBlock) void sim_order_scatter_kernel(uint32_t n_cfg, SimWs ws) {
    const uint32_t c = blockIdx.x * kBlock + threadIdx.x;
    if (c < n_cfg) ws.perm[atomicAdd(&ws.bins[ws.bucket[c]], 1u)] = c;
}

__global__ __launch_bounds__(kKeyBins) void sim_order_clear_kernel(SimWs ws) { ws.bins[threadIdx.x] = 0; }

// Heap of the decoders' finishing steps, one per lane.  Node 0 lives in a register, nodes 1 .. cap in the lane's
// segment of LDS, deeper nodes in global memory.  4-ary: the children of node i are 4i+1 .. 4i+4.
// Key = finishing step << 10 | request; 32-bit keys when every finishing step fits 22 bits (twice the nodes in LDS).
template <typename KeyT>
struct LaneHeap {
    KeyT top;
    KeyT *lds;            // node i (1 <= i <= cap) at lds[i - 1]
    KeyT *mem;            // node i (i > cap) at mem[i]
    uint32_t cap, n;
    __device__ KeyT get(uint32_t i) const { return i <= cap ? lds[i - 1] : mem[i]; }
    __device__ void set(uint32_t i, KeyT k) {
        if (i <= cap) lds[i - 1] = k; else mem[i] = k;
    }
    __device__ void push(KeyT key) {                // the new node rises from the end
        uint32_t i = n++;
        while (i > 0) {
            const uint32_t par = (i - 1) >> 2;
            const KeyT pk = par == 0 ? top : get(par);
            if (pk <= key) break;
            set(i, pk);
            i = par;
        }
        if (i == 0) top = key; else set(i, key);
    }
    __device__ void pop() {                         // the last node sinks from the root
        --n;
        if (n == 0) {
            top = (KeyT)~(KeyT)0;
            return;
        }
        const KeyT last = get(n);
        uint32_t i = 0;
        for (;;) {
            const uint32_t c0 = 4 * i + 1;
            if (c0 >= n) break;
            KeyT k[4];
#pragma unroll
            for (uint32_t j = 0; j < 4; ++j) k[j] = get(c0 + j < n ? c0 + j : c0);      // all four requested at once
            KeyT best = k[0];
            uint32_t bi = c0;
#pragma unroll
            for (uint32_t j = 1; j < 4; ++j)
                if (c0 + j < n && k[j] < best) { best = k[j]; bi = c0 + j; }
            if (best >= last) break;
            if (i == 0) top = best; else set(i, best);
            i = bi;
        }
        if (i == 0) top = last; else set(i, last);
    }
};

// Time of r consecutive decode-only steps of T decoders whose total context is C0 before the first one:
// r * (everything but attention) + L * (attention over contexts C0, C0 + T, ..), the latter in closed form.
template <bool ADDITIVE>
__device__ inline double run_time(const TimeCoef &tc, double step_const, double T, double r_T, double C0, double r) {
    const double att = attention_series<ADDITIVE>(tc.c_att, tc.m_att_k, T * tc.m_att_t, C0 - T, T, r_T, r);
    return fma(r, step_const, tc.L * att);
}

// CLOSED_RUNS: runs of decode-only steps are advanced by run_time() in one go (GUIDE_SIM_CLOSED_FORM_RUNS);
// otherwise step by step with the general step's own arithmetic.
// ordered: configurations run in the order ws.perm (longest expected first); otherwise as given.
// heap_slots: keys that the LDS behind the staged tables holds for the whole block; they are shared out among the
// block's lanes in proportion to the most decoders each can have (its sequence cap), so that a lane that can
// run a thousand sequences gets a long segment and a lane capped at four next to nothing.
template <bool ADDITIVE, bool PREFILL_FIRST, bool CLOSED_RUNS, typename KeyT>
__global__ __launch_bounds__(kSimBlock) void simulate_kernel(GridDesc g, const DevTables *__restrict__ tab,
                                                             const TraceDev *__restrict__ trace, uint32_t n_req,
                                                             const uint32_t *__restrict__ cfg_idx,
                                                             const double *__restrict__ rate_in, uint32_t n_cfg,
                                                             guide_sim_out out, SimWs ws, uint32_t max_run,
                                                             uint32_t heap_slots, uint32_t ordered) {
    extern __shared__ __align__(16) unsigned char s_raw[];
    SimLds &s = *(SimLds *)s_raw;
    KeyT *s_heap = (KeyT *)(s_raw + sizeof(SimLds));
    __shared__ uint32_t s_cap[kSimBlock], s_off[kSimBlock];
    __shared__ uint32_t s_total[kSimBlock / kWave];
    for (uint32_t i = threadIdx.x; i < kNumAxes * GUIDE_MAX_AXIS_VALUES; i += blockDim.x)
        (&s.axis[0][0])[i] = (&tab->axis_vals[0][0])[i];
    for (uint32_t i = threadIdx.x; i < g.n_models * 8u; i += blockDim.x)
        ((uint32_t *)s.models)[i] = ((const uint32_t *)tab->models)[i];
    for (uint32_t i = threadIdx.x; i < n_req; i += blockDim.x) {
        s.arrival[i] = trace->arrival[i];
        s.n_in[i] = trace->n_in[i];
        s.n_out[i] = trace->n_out[i];
    }
    __syncthreads();
    const uint32_t pos = blockIdx.x * kSimBlock + threadIdx.x;     // launch position
    const bool in_range = pos < n_cfg;
    const uint32_t c = in_range ? (ordered ? ws.perm[pos] : pos) : 0u;      // its configuration

    uint32_t v[kNumAxes];
    bool alive = false;                                           // this lane has a simulation to run
    uint32_t max_seqs = 1, blk = 1, mbt = 1;
    double rate = 1.0, c_avail = 0.0, tokens = 0.0;
    uint64_t step_bound = n_req;
    long long n_blk = 0;
    Coef cf;
    TimeCoef tc;
    Div32 dblk = make_div32(1);
    // KV blocks of a request of `tok` >= 1 tokens: ceil(tok / blk) without the 32-bit overflow of tok + blk - 1
    auto blocks_of = [&](uint32_t tok) { return (long long)div32(tok - 1, dblk) + 1; };
    if (in_range) {
        const bool bad_index = decode_sim_index(s.axis, g, cfg_idx[c], v);
        max_seqs = v[AX_BATCH]; blk = v[AX_BLK]; mbt = v[AX_MBT];
        const guide_hw hw = tab->hw[v[AX_HW]];
        rate = rate_in[c];
        cf = make_coef(s.models[v[AX_MODEL]], v[AX_TP], v[AX_WBITS]);
        tc = make_time_coef(cf, 1.0 / hw.peak_flops, 1.0 / hw.hbm_bw, 1.0 / hw.link_bw, hw.link_lat);
        dblk = make_div32(blk);
        // KV pool in blocks; every request must fit on its own
        c_avail = hw.cap_bytes - cf.w_gpu;
        uint32_t max_tok = 0;
        for (uint32_t i = 0; i < n_req; ++i) {
            const uint32_t t = s.n_in[i] + s.n_out[i];
            max_tok = t > max_tok ? t : max_tok;
            step_bound += t;
            tokens += (double)s.n_out[i];
        }
        if (c_avail > 0.0) {
            const double nb = floor(c_avail / ((double)blk * cf.kv_tok));
            n_blk = nb >= 9.0e18 ? 0x7FFFFFFFFFFFFFFFll : (long long)nb;
        }
        if (bad_index || !(c_avail > 0.0) || blocks_of(max_tok) > n_blk || !(rate > 0.0)) {
            out.ttft_p50[c] = INFINITY; out.ttft_p99[c] = INFINITY; out.mean_tpot[c] = INFINITY; out.tokens_s[c] = 0.0;
            out.status[c] = (bad_index || !(rate > 0.0)) ? GUIDE_SIM_BAD_INPUT : GUIDE_SIM_INFEASIBLE;
            out.n_steps[c] = 0; out.n_request_steps[c] = 0;
        } else {
            alive = true;
        }
    }

    // LDS segments of the heaps: a lane can have at most min(sequence cap, requests) decoders, one of them in a
    // register; when the block's lanes want more than the LDS holds, every segment shrinks by the same factor
    const uint32_t want = alive ? (max_seqs < n_req ? max_seqs : n_req) - 1u : 0u;
    {
        uint32_t t = want;
        for (int off = kWave / 2; off > 0; off >>= 1) t += __shfl_xor(t, off, kWave);
        if (threadIdx.x % kWave == 0) s_total[threadIdx.x / kWave] = t;
        __syncthreads();
        uint32_t total = 0;
        for (uint32_t w = 0; w < kSimBlock / kWave; ++w) total += s_total[w];
        uint32_t cap = want;
        if (total > heap_slots) cap = (uint32_t)((double)want * ((double)heap_slots / (double)total) * (1.0 - 0x1p-30));
        s_cap[threadIdx.x] = cap;
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t run = 0;
            for (uint32_t i = 0; i < kSimBlock; ++i) {
                s_off[i] = run;
                run += s_cap[i];
            }
        }
        __syncthreads();
    }
    if (!alive) return;

    LaneHeap<KeyT> heap;
    heap.top = (KeyT)~(KeyT)0;
    heap.lds = s_heap + s_off[threadIdx.x];
    heap.mem = (KeyT *)(ws.heap + (size_t)pos * n_req);
    heap.cap = s_cap[threadIdx.x];
    heap.n = 0;
    double *first = ws.first + (size_t)c * n_req, *fin = ws.fin + (size_t)c * n_req;

    double now = 0.0, max_fin = -INFINITY;
    uint32_t next = 0, pf_head = 0, pf_done = 0, n_dec = 0, n_done = 0;
    uint64_t s_ctx = 0, step = 0, dstep = 0, n_rs = 0;   // dstep counts the steps in which decoders ran
    long long free_blk = n_blk;
    uint32_t status = GUIDE_SIM_OK;
    double arr_next = s.arrival[0] / rate;   // arrival time of request `next`
    long long need_next = blocks_of(s.n_in[0] + s.n_out[0]);
    double kept_base = 0.0, kept_lm = 0.0;   // layer_base / lm_head for kept_dec decode tokens (a pure function of the count)
    uint32_t kept_dec = 0;

    while (n_done < n_req) {
        // Run of decode-only steps: no prompt is waiting for chunks, and nothing changes until the first
        // decoder finishes or a request that could be admitted arrives.
        if (pf_head == next && n_dec > 0) {
            if (kept_dec != n_dec) {
                kept_base = layer_base<ADDITIVE>(tc, (double)n_dec);
                kept_lm = lm_head<ADDITIVE>(tc, (double)n_dec);
                kept_dec = n_dec;
            }
            const bool can_admit = next < n_req && n_dec < max_seqs && need_next <= free_blk;
            const double arr_stop = can_admit ? arr_next : INFINITY;
            const uint64_t stop = (uint64_t)(heap.top >> 10); // the step whose book-keeping retires a decoder
            // steps left before that one (stop > dstep: its last token is still to come)
            const uint64_t left = stop - dstep - 1;
            const double T = (double)n_dec;
            double ctx = (double)s_ctx;                       // integers below 2^53: exact in fp64
            uint32_t run = 0;
            if (CLOSED_RUNS) {
                // The run takes r = min(left, least r with arrival <= now + time of r steps) steps.  The search
                // walks up from r = 0 without overshooting: the steps still to come each take at most the time
                // of the last one that could be needed, so floor(remaining / that) of them fit for sure.
                const uint32_t r_max = left < 0x40000000ull ? (uint32_t)left : 0x40000000u;
                const double step_const = fma(tc.L, kept_base, kept_lm), r_T = fast_recip(T);
                auto t_at = [&](double j) {
                    const double cj = fma(j, T, ctx);
                    return fma(tc.L, attention<ADDITIVE>(tc, T, cj, cj), step_const);
                };
                double s_run = 0.0;
                if (!can_admit) {
                    run = r_max;
                    s_run = run_time<ADDITIVE>(tc, step_const, T, r_T, ctx, (double)run);
                } else {
                    for (;;) {
                        const double rem = arr_stop - (now + s_run);
                        if (!(rem > 0.0) || run == r_max) break;
                        const double room = (double)(r_max - run);
                        const double ub = fmin(ceil(rem * fast_recip(t_at((double)run))), room);
                        const double t_hi = t_at((double)run + fmax(ub, 1.0) - 1.0);
                        const double q = fmin(fmax(floor(rem * fast_recip(t_hi)), 1.0), room);
                        run += (uint32_t)q;
                        s_run = run_time<ADDITIVE>(tc, step_const, T, r_T, ctx, (double)run);
                    }
                }
                now += s_run;
            } else {
                const uint32_t r_cap = left < max_run ? (uint32_t)left : max_run;
                auto step_time = [&](double cj) { return fma(tc.L, kept_base + attention<ADDITIVE>(tc, T, cj, cj), kept_lm); };
                // Four steps at a time without a branch between them: the times after each step are formed in
                // step order (n1 = now + t1, n2 = n1 + t2, ..), and the run stops after the first k steps whose
                // starting time is still before the arrival -- times only grow, so k is a count of compares.
                // Each step is the general step below with its invariant parts left out: the same operations
                // in the same order on the same values.
                bool go = true;
                while (go && run + 4 <= r_cap) {
                    const double c2 = ctx + T, c3 = c2 + T, c4 = c3 + T;
                    const double n1 = now + step_time(ctx), n2 = n1 + step_time(c2), n3 = n2 + step_time(c3),
                                 n4 = n3 + step_time(c4);
                    const uint32_t k = arr_stop <= now ? 0u : arr_stop <= n1 ? 1u : arr_stop <= n2 ? 2u : arr_stop <= n3 ? 3u : 4u;
                    now = k == 0 ? now : k == 1 ? n1 : k == 2 ? n2 : k == 3 ? n3 : n4;
                    ctx = k == 0 ? ctx : k == 1 ? c2 : k == 2 ? c3 : k == 3 ? c4 : c4 + T;
                    run += k;
                    go = k == 4;
                }
                while (go && run < r_cap && !(arr_stop <= now)) {
                    now += step_time(ctx);
                    ctx += T;
                    ++run;
                }
            }
            step += run;
            dstep += run;
            n_rs += (uint64_t)run * n_dec;
            s_ctx += (uint64_t)run * n_dec;
        }
        uint32_t n_active = (next - pf_head) + n_dec;
        // 1. idle jump to the next arrival
        if (n_active == 0 && next < n_req) now = arr_next > now ? arr_next : now;
        // 2. FCFS admission; stop at the first request that cannot enter
        while (next < n_req && n_active < max_seqs && arr_next <= now && need_next <= free_blk) {
            free_blk -= need_next;
            ++next;
            ++n_active;
            if (next < n_req) {
                arr_next = s.arrival[next] / rate;
                need_next = blocks_of(s.n_in[next] + s.n_out[next]);
            } else {
                arr_next = INFINITY;
            }
        }
        // 3. schedule.  Split-fuse: one token per decoder, then prompt chunks in admission order under
        // the remaining budget.  Prefill-first: while prompts wait, whole prompts only (as many as fit the
        // budget, the first always) and the decoders pause.
        const bool decoders_run = !(PREFILL_FIRST && pf_head < next);
        double T = 0.0, Q = 0.0, K = 0.0, n_lm = 0.0;
        if (decoders_run) {
            T = (double)n_dec; Q = (double)s_ctx; K = (double)s_ctx; n_lm = (double)n_dec;
        }
        long long budget = (long long)mbt - (long long)n_dec;
        uint32_t h = pf_head, done = pf_done, chunks = 0;
        if (PREFILL_FIRST) {
            long long used = 0;
            while (h < next && (chunks == 0 || used + (long long)s.n_in[h] <= (long long)mbt)) {
                const double len = (double)s.n_in[h];
                used += (long long)s.n_in[h];
                T += len;
                Q = fma(len, len, Q);
                K += len;
                n_lm += 1.0;
                ++chunks;
                ++h;
            }
            budget = 0;
        }
        while (h < next && budget > 0) {
            const long long rem = (long long)(s.n_in[h] - done);
            const long long ch = rem < budget ? rem : budget;
            budget -= ch;
            const double C = (double)ch, ctx = (double)(done + (uint32_t)ch);
            T += C;
            Q = fma(C, ctx, Q);
            K += ctx;
            ++chunks;
            if (ch == rem) {
                n_lm += 1.0;
                ++h;
                done = 0;
            } else {
                done += (uint32_t)ch;
            }
        }
        // 4. one engine step.  A step with decode tokens only repeats the previous step's token count
        // unless a request joined or left, so the part of the pass that depends on the token count alone
        // is kept from step to step (same operations, same rounding, as evaluating the whole pass)
        if (chunks == 0) {
            if (n_dec != kept_dec) {
                kept_base = layer_base<ADDITIVE>(tc, T);
                kept_lm = lm_head<ADDITIVE>(tc, n_lm);
                kept_dec = n_dec;
            }
            now += fma(tc.L, kept_base + attention<ADDITIVE>(tc, T, Q, K), kept_lm);
        } else {
            now += pass_time<ADDITIVE>(tc, T, Q, K, n_lm);
        }
        ++step;
        n_rs += (decoders_run ? n_dec : 0u) + chunks;
        // 5. book-keeping: decoders emitted a token; those at their last one leave
        if (decoders_run) {
            ++dstep;
            s_ctx += n_dec;
        }
        while (decoders_run && heap.n > 0 && (uint64_t)(heap.top >> 10) == dstep) {
            const uint32_t r = (uint32_t)(heap.top & 1023u);
            heap.pop();
            const uint32_t r_tok = s.n_in[r] + s.n_out[r];
            free_blk += blocks_of(r_tok);
            --n_dec;
            s_ctx -= (uint64_t)r_tok;
            ++n_done;
            fin[r] = now;
            max_fin = now;
        }
        // prompts completed in this step emit their first token
        for (uint32_t r = pf_head; r < h; ++r) {
            const uint32_t r_in = s.n_in[r], r_out = s.n_out[r];
            first[r] = now;
            if (r_out == 1) {
                free_blk += blocks_of(r_in + 1);
                ++n_done;
                fin[r] = now;
                max_fin = now;
            } else {
                ++n_dec;
                s_ctx += (uint64_t)r_in + 1;
                heap.push((KeyT)(((dstep + r_out - 1) << 10) | r));
            }
        }
        pf_head = h;
        pf_done = done;
        if (step > step_bound) {   // every step consumes at least one token of some request
            status = GUIDE_SIM_INTERNAL;
            break;
        }
    }

    out.tokens_s[c] = status == GUIDE_SIM_OK ? tokens / (max_fin - s.arrival[0] / rate) : 0.0;
    out.status[c] = status;
    out.n_steps[c] = step;
    out.n_request_steps[c] = n_rs;
    if (status != GUIDE_SIM_OK) {
        out.ttft_p50[c] = INFINITY; out.ttft_p99[c] = INFINITY; out.mean_tpot[c] = INFINITY;
    }
}

// One wave per simulated configuration that ended normally.  TTFT of request i = first token time - arrival /
// rate; the 1024 values (absent requests count as +inf) are sorted inside the wave's registers, 16 per lane, by
// a bitonic network in which every compare-exchange puts the smaller value at the smaller index: element
// e = 16 * lane + register; a stage pairs e with e ^ m, which is another register of the same lane while m < 16
// and the same-numbered (or mirrored) register of lane ^ (m / 16) otherwise.  Then nearest-rank
// p50 = sorted[ceil(n/2) - 1] and p99 = sorted[ceil(0.99 n) - 1]; mean TPOT = mean over requests with more than
// one token of (finish - first token) / (tokens - 1).
constexpr uint32_t kPerLane = GUIDE_MAX_REQUESTS / kWave;       // 16
static_assert(kPerLane == 16, "the network below is written for 16 values per lane");

constexpr uint32_t top_bit(uint32_t x) { return x < 2 ? x : 2 * top_bit(x / 2); }
// compare-exchange inside a lane: the smaller value to the smaller register
__device__ inline void cx(double &a, double &b) {
    const double lo = fmin(a, b), hi = fmax(a, b);
    a = lo;
    b = hi;
}
// One stage of the network.  MASK: the xor mask on element numbers.
template <uint32_t MASK>
__device__ inline void sort_stage(double (&v)[kPerLane], uint32_t lane) {
    if constexpr (MASK < kPerLane) {
#pragma unroll
        for (uint32_t r = 0; r < kPerLane; ++r)
            if ((r ^ MASK) > r) cx(v[r], v[r ^ MASK]);
    } else {
        constexpr uint32_t kLaneMask = MASK / kPerLane, kRegMask = MASK % kPerLane;     // kRegMask: 0 or 15 (mirror)
        // this lane holds the smaller indices of its pairs when the top bit of the lane mask is clear in its number
        constexpr uint32_t kTop = top_bit(kLaneMask);
        const bool keep_min = (lane & kTop) == 0;
        double o[kPerLane];
#pragma unroll
        for (uint32_t r = 0; r < kPerLane; ++r) o[r] = __shfl_xor(v[r ^ kRegMask], (int)kLaneMask, kWave);
#pragma unroll
        for (uint32_t r = 0; r < kPerLane; ++r) v[r] = keep_min ? fmin(v[r], o[r]) : fmax(v[r], o[r]);
    }
}
// Merge of sorted runs of K / 2 elements into sorted runs of K: the mirror stage, then halving distances.
template <uint32_t K>
__device__ inline void sort_merge(double (&v)[kPerLane], uint32_t lane) {
    sort_stage<K - 1>(v, lane);
    if constexpr (K >= 4) sort_stage<K / 4>(v, lane);
    if constexpr (K >= 8) sort_stage<K / 8>(v, lane);
    if constexpr (K >= 16) sort_stage<K / 16>(v, lane);
    if constexpr (K >= 32) sort_stage<K / 32>(v, lane);
    if constexpr (K >= 64) sort_stage<K / 64>(v, lane);
    if constexpr (K >= 128) sort_stage<K / 128>(v, lane);
    if constexpr (K >= 256) sort_stage<K / 256>(v, lane);
    if constexpr (K >= 512) sort_stage<K / 512>(v, lane);
    if constexpr (K >= 1024) sort_stage<K / 1024>(v, lane);
}
// element `e` of the sorted sequence, in every lane
__device__ inline double sorted_at(const double (&v)[kPerLane], uint32_t e) {
    double x = v[0];
#pragma unroll
    for (uint32_t r = 1; r < kPerLane; ++r) x = (e % kPerLane) == r ? v[r] : x;
    return __shfl(x, (int)(e / kPerLane), kWave);
}

__global__ __launch_bounds__(kPctBlock) void percentile_kernel(SimWs ws, const TraceDev *__restrict__ trace,
                                                               const double *__restrict__ rate_in, uint32_t n_req,
                                                               uint32_t n_cfg, guide_sim_out out) {
    const uint32_t lane = threadIdx.x % kWave;
    const uint32_t c = blockIdx.x * (kPctBlock / kWave) + threadIdx.x / kWave;      // wave-uniform
    if (c >= n_cfg || out.status[c] != GUIDE_SIM_OK) return;
    const double rate = rate_in[c];
    const double *first = ws.first + (size_t)c * n_req, *fin = ws.fin + (size_t)c * n_req;
    double v[kPerLane];
    double tp = 0.0;
    uint32_t n_tp = 0;
#pragma unroll
    for (uint32_t r = 0; r < kPerLane; ++r) {
        const uint32_t i = r * kWave + lane;                // coalesced; the sort does not care where a value starts
        double t = INFINITY;
        if (i < n_req) {
            const double f = first[i];
            t = f - trace->arrival[i] / rate;
            const uint32_t n_out = trace->n_out[i];
            if (n_out > 1) {
                tp += (fin[i] - f) / (double)(n_out - 1);
                ++n_tp;
            }
        }
        v[r] = t;
    }
    for (int off = kWave / 2; off > 0; off >>= 1) {
        tp += __shfl_xor(tp, off, kWave);
        n_tp += __shfl_xor(n_tp, off, kWave);
    }
    sort_merge<2>(v, lane);
    sort_merge<4>(v, lane);
    sort_merge<8>(v, lane);
    sort_merge<16>(v, lane);
    sort_merge<32>(v, lane);
    sort_merge<64>(v, lane);
    sort_merge<128>(v, lane);
    sort_merge<256>(v, lane);
    sort_merge<512>(v, lane);
    sort_merge<1024>(v, lane);
    const double p50 = sorted_at(v, (n_req + 1) / 2 - 1);
    const double p99 = sorted_at(v, (uint32_t)((99ull * n_req + 99) / 100 - 1));
    if (lane == 0) {
        out.ttft_p50[c] = p50;
        out.ttft_p99[c] = p99;
        out.mean_tpot[c] = n_tp ? tp / (double)n_tp : 0.0;
    }
}

}  // namespace

size_t simulate_workspace_bytes(uint32_t n_cfg, uint32_t n_req) {
    return (size_t)n_cfg * n_req * 24 + (size_t)n_cfg * 8 + kKeyBins * 4 + 256;
}

hipError_t launch_simulate(const GridDesc &g, const DevTables *tab, const TraceDev *trace, uint32_t n_req,
                           const uint32_t *cfg_idx, const double *rate, uint32_t n_cfg, bool additive,
                           bool prefill_first, bool closed_runs, const guide_sim_out &out, void *ws_, hipStream_t stream,
                           double sum_in, double sum_out) {
    const SimWs ws = sim_ws(ws_, n_cfg, n_req);
    // Stepped runs: lanes wait for the longest run of their wave before the next general step, so runs are
    // capped (64 steps measured best among 4..1024 on the 65 536-configuration mix; stopping a run once few
    // lanes of the wave are still in it measured worse at every setting tried).
    const uint32_t max_run = 64;
    // LDS beyond the staged tables holds heap nodes of the block's lanes; 32-bit keys when every finishing step
    // (at most the trace's generated tokens) fits 22 bits
    const bool key32 = sum_out < 4194303.0;
    const size_t key_bytes = key32 ? sizeof(uint32_t) : sizeof(uint64_t);
    int dev = 0, lds_max = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
    if (e != hipSuccess) return e;
    const size_t fixed = sizeof(SimLds) + kSimStaticLds;
    if ((size_t)lds_max < fixed) return hipErrorInvalidValue;
    size_t heap_bytes = (size_t)lds_max - fixed;
    const size_t most = (size_t)kSimBlock * n_req * key_bytes;          // no lane needs more than n_req - 1 nodes
    heap_bytes = heap_bytes < most ? heap_bytes : most;
    heap_bytes -= heap_bytes % 16;
    const uint32_t heap_slots = (uint32_t)(heap_bytes / key_bytes);
    const size_t lds_bytes = sizeof(SimLds) + heap_bytes;
    const dim3 grid((n_cfg + kSimBlock - 1) / kSimBlock), block(kSimBlock);
    const dim3 ogrid((n_cfg + kBlock - 1) / kBlock), oblock(kBlock);
    // Stepped runs: configurations run longest first, so that the lanes of a wave end together.  With closed-form
    // runs every lane does about the same number of rounds (one per event), and the order given mixes lanes with
    // short and long heaps in a block, which is what the shared LDS wants.
    const uint32_t ordered = closed_runs ? 0u : 1u;
    if (ordered) {
        hipLaunchKernelGGL(sim_order_clear_kernel, dim3(1), dim3(kKeyBins), 0, stream, ws);
        if (additive)
            hipLaunchKernelGGL(sim_order_count_kernel<true>, ogrid, oblock, 0, stream, g, tab, n_req, cfg_idx, rate, n_cfg, ws, sum_in, sum_out);
        else
            hipLaunchKernelGGL(sim_order_count_kernel<false>, ogrid, oblock, 0, stream, g, tab, n_req, cfg_idx, rate, n_cfg, ws, sum_in, sum_out);
        hipLaunchKernelGGL(sim_order_scan_kernel, dim3(1), dim3(kKeyBins), 0, stream, ws);
        hipLaunchKernelGGL(sim_order_scatter_kernel, ogrid, oblock, 0, stream, n_cfg, ws);
    }
    const int variant = (additive ? 8 : 0) | (prefill_first ? 4 : 0) | (closed_runs ? 2 : 0) | (key32 ? 1 : 0);
#define GUIDE_SIM(A, P, C, K32)                                                                                    \
    case ((A ? 8 : 0) | (P ? 4 : 0) | (C ? 2 : 0) | (K32 ? 1 : 0)): {                                               \
        auto kern = simulate_kernel<A, P, C, std::conditional<K32, uint32_t, uint64_t>::type>;                      \
        e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);    \
        if (e != hipSuccess) return e;                                                                              \
        hipLaunchKernelGGL(kern, grid, block, lds_bytes, stream, g, tab, trace, n_req, cfg_idx, rate, n_cfg, out, ws, \
                           max_run, heap_slots, ordered);                                                           \
        break;                                                                                                      \
    }
    switch (variant) {
        GUIDE_SIM(false, false, false, false) GUIDE_SIM(false, false, false, true) GUIDE_SIM(false, false, true, false)
        GUIDE_SIM(false, false, true, true) GUIDE_SIM(false, true, false, false) GUIDE_SIM(false, true, false, true)
        GUIDE_SIM(false, true, true, false) GUIDE_SIM(false, true, true, true) GUIDE_SIM(true, false, false, false)
        GUIDE_SIM(true, false, false, true) GUIDE_SIM(true, false, true, false) GUIDE_SIM(true, false, true, true)
        GUIDE_SIM(true, true, false, false) GUIDE_SIM(true, true, false, true) GUIDE_SIM(true, true, true, false)
        GUIDE_SIM(true, true, true, true)
    }
#undef GUIDE_SIM
    hipLaunchKernelGGL(percentile_kernel, dim3((n_cfg + kPctBlock / kWave - 1) / (kPctBlock / kWave)), dim3(kPctBlock), 0,
                       stream, ws, trace, rate, n_req, n_cfg, out);
    return hipGetLastError();
}

}  // namespace guide
