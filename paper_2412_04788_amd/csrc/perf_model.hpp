// Device-side performance model: per-operator FLOPs / bytes of one decoder
// layer, roofline pass time, static-batch prefill, closed-form decode series and
// KV-memory feasibility.  One candidate configuration per lane.
//
// Paper sections followed: Parallel Simulator "Task and GPU Models" (a task is a
// compute load and a data size; a GPU is compute performance, memory bandwidth,
// communication bandwidth, latency), "Roofline Model for Performance Analysis",
// "Time Calculation"; Model Analyzer "Dynamic Batch Size Adjustment" and
// "Dynamic Sequence Length Adjustment"; Inference Engine Steps 1 and 2.
#pragma once

#include "common.hpp"

namespace guide {

constexpr double kActBytes = 2.0;  // bytes per activation element
constexpr double kKvBytes = 2.0;   // bytes per cached K or V element

enum { OP_QKV = 0, OP_OPROJ, OP_UP, OP_DOWN, OP_ROUTER, N_LINEAR };

// Work of one GPU's share of the model, per unit of the pass descriptors
// (T tokens, Q query-context pairs, K cached tokens, n_lm LM-head rows).
struct Coef {
    double L;
    double f[N_LINEAR];   // FLOPs per token
    double w[N_LINEAR];   // weight bytes per pass (UP/DOWN: per expert whose weights are read)
    double a[N_LINEAR];   // activation bytes per token
    double f_att, a_att, c_att;   // attention: FLOPs per pair, bytes per token, bytes per cached token
    double a_nm;                  // two norms: bytes per token
    double f_lm, w_lm, a_lm;      // LM head per row
    double m_ar, n_ar;            // all-reduce: link bytes per token (ring factor folded in), latency hops
    double w_gpu, kv_tok, p_total;
    double E, k;
};

// The same, multiplied by the hardware's reciprocals: seconds per unit.
struct TimeCoef {
    double L;
    double c[N_LINEAR], m0[N_LINEAR], m1[N_LINEAR];
    double c_att, m_att_t, m_att_k;
    double m_nm;
    double c_lm, m0_lm, m1_lm;
    double ar1, ar0;
    double E, k;
};

struct HwRecip {
    double r_peak, r_bw, cap, r_link, lat;
};

// rp = 1 / p_ (correctly rounded).
__device__ inline Coef make_coef(const guide_model &md, uint32_t p_, uint32_t wbits, double rp) {
    Coef c;
    const double p = (double)p_, w = (double)wbits * 0.125, a = kActBytes;
    const double d = (double)md.d, dh = (double)(md.d / md.n_h);
    const double dq = (double)md.n_h * dh, dkv = (double)md.n_kv * dh;
    const double dff = (double)md.d_ff, V = (double)md.V, E = (double)md.E, k = (double)md.k;
    const double gkv = (double)((md.n_kv + p_ - 1) / p_) * dh;   // KV heads replicate when n_kv < p
    const double pf1 = 2.0 * d * dff, pf2 = dff * d, prt = md.E > 1 ? d * E : 0.0;
    const double pattn = d * dq + 2.0 * d * dkv + dq * d;
    c.L = (double)md.L;
    c.f[OP_QKV] = 2.0 * d * (dq + 2.0 * dkv) * rp;
    c.w[OP_QKV] = w * d * (dq + 2.0 * dkv) * rp;
    c.a[OP_QKV] = a * d + a * (dq + 2.0 * dkv) * rp;
    c.f_att = 4.0 * dq * rp;
    c.a_att = 2.0 * a * dq * rp;
    c.c_att = 2.0 * kKvBytes * gkv;
    c.f[OP_OPROJ] = 2.0 * dq * d * rp;
    c.w[OP_OPROJ] = w * dq * d * rp;
    c.a[OP_OPROJ] = a * dq * rp + a * d;
    c.f[OP_UP] = 2.0 * k * pf1 * rp;
    c.w[OP_UP] = w * pf1 * rp;
    c.a[OP_UP] = a * d + 2.0 * a * k * dff * rp;
    c.f[OP_DOWN] = 2.0 * k * pf2 * rp;
    c.w[OP_DOWN] = w * pf2 * rp;
    c.a[OP_DOWN] = a * k * dff * rp + a * d;
    c.f[OP_ROUTER] = 2.0 * prt;                       // router is replicated on every GPU
    c.w[OP_ROUTER] = w * prt;
    c.a[OP_ROUTER] = md.E > 1 ? a * d + a * E : 0.0;
    c.a_nm = 4.0 * a * d;
    c.f_lm = 2.0 * d * V * rp;
    c.w_lm = w * d * V * rp;
    c.a_lm = a * d + a * V * rp;
    c.m_ar = p_ > 1 ? 2.0 * (p - 1.0) * rp * (a * d) : 0.0;
    c.n_ar = p_ > 1 ? 2.0 * (p - 1.0) : 0.0;
    c.p_total = c.L * (pattn + E * (pf1 + pf2) + prt) + 2.0 * V * d;
    c.w_gpu = w * c.p_total / p;                       // same operation order as a plain evaluator
    c.kv_tok = 2.0 * c.L * gkv * kKvBytes;
    c.E = E;
    c.k = k;
    return c;
}

__device__ inline Coef make_coef(const guide_model &md, uint32_t p_, uint32_t wbits) {
    return make_coef(md, p_, wbits, 1.0 / (double)p_);
}

// r_peak / r_bw already include the efficiency sample.
__device__ inline TimeCoef make_time_coef(const Coef &c, double r_peak, double r_bw, double r_link, double lat) {
    TimeCoef t;
    t.L = c.L;
#pragma unroll
    for (int i = 0; i < N_LINEAR; ++i) {
        t.c[i] = c.f[i] * r_peak;
        t.m0[i] = c.w[i] * r_bw;
        t.m1[i] = c.a[i] * r_bw;
    }
    t.c_att = c.f_att * r_peak;
    t.m_att_t = c.a_att * r_bw;
    t.m_att_k = c.c_att * r_bw;
    t.m_nm = c.a_nm * r_bw;
    t.c_lm = c.f_lm * r_peak;
    t.m0_lm = c.w_lm * r_bw;
    t.m1_lm = c.a_lm * r_bw;
    t.ar1 = c.m_ar * r_link;
    t.ar0 = c.n_ar * lat;
    t.E = c.E;
    t.k = c.k;
    return t;
}

template <bool ADDITIVE>
__device__ inline double op_time(double t_compute, double t_memory) {
    return ADDITIVE ? t_compute + t_memory : fmax(t_compute, t_memory);
}

// Sum of the layer ops that do not depend on the attention workload, plus the
// norms and the two all-reduces: everything of a layer but attention.
template <bool ADDITIVE>
__device__ inline double layer_base(const TimeCoef &t, double T) {
    const double eld = fmin(t.E, t.k * T);   // experts whose weights are read
    double s = op_time<ADDITIVE>(T * t.c[OP_QKV], fma(T, t.m1[OP_QKV], t.m0[OP_QKV]));
    s += op_time<ADDITIVE>(T * t.c[OP_OPROJ], fma(T, t.m1[OP_OPROJ], t.m0[OP_OPROJ]));
    s += op_time<ADDITIVE>(T * t.c[OP_UP], fma(T, t.m1[OP_UP], eld * t.m0[OP_UP]));
    s += op_time<ADDITIVE>(T * t.c[OP_DOWN], fma(T, t.m1[OP_DOWN], eld * t.m0[OP_DOWN]));
    s += op_time<ADDITIVE>(T * t.c[OP_ROUTER], fma(T, t.m1[OP_ROUTER], t.m0[OP_ROUTER]));
    s += T * t.m_nm;
    s += 2.0 * fma(T, t.ar1, t.ar0);
    return s;
}

template <bool ADDITIVE>
__device__ inline double lm_head(const TimeCoef &t, double n_lm) {
    return n_lm > 0.0 ? op_time<ADDITIVE>(n_lm * t.c_lm, fma(n_lm, t.m1_lm, t.m0_lm)) : 0.0;
}

template <bool ADDITIVE>
__device__ inline double attention(const TimeCoef &t, double T, double Q, double K) {
    return op_time<ADDITIVE>(Q * t.c_att, fma(K, t.m_att_k, T * t.m_att_t));
}

// t_pass = L * (layer ops + 2 all-reduces) + LM head.
template <bool ADDITIVE>
__device__ inline double pass_time(const TimeCoef &t, double T, double Q, double K, double n_lm) {
    return fma(t.L, layer_base<ADDITIVE>(t, T) + attention<ADDITIVE>(t, T, Q, K), lm_head<ADDITIVE>(t, n_lm));
}

// Static batch of b prompts of s tokens under a budget of mbt tokens per pass.
template <bool ADDITIVE>
__device__ inline double prefill_time(const TimeCoef &t, uint32_t b, uint32_t s, uint32_t mbt) {
    if (s <= mbt) {
        uint32_t r = mbt / s;
        r = r < b ? r : b;
        const uint32_t n_full = b / r, rem = b - n_full * r;
        const double S = (double)s;
        double R = (double)r;
        double total = (double)n_full * pass_time<ADDITIVE>(t, R * S, R * S * S, R * S, R);
        if (rem > 0) {
            R = (double)rem;
            total += pass_time<ADDITIVE>(t, R * S, R * S * S, R * S, R);
        }
        return total;
    }
    // prompt longer than the budget: ceil(s / mbt) segments per request, requests one after another
    const uint32_t n_seg = (s + mbt - 1) / mbt;
    double one = 0.0;
    for (uint32_t j = 0; j < n_seg; ++j) {
        uint32_t c = s - j * mbt;
        c = c < mbt ? c : mbt;
        const double C = (double)c, ctx = (double)(j * mbt + c);
        one += pass_time<ADDITIVE>(t, C, C * ctx, ctx, j == n_seg - 1 ? 1.0 : 0.0);
    }
    return (double)b * one;
}

// sum_{j=j0+1}^{j1} (s + j)
__device__ inline double ctx_sum(double s, double j0, double j1) {
    return (j1 - j0) * s + 0.5 * (j1 * (j1 + 1.0) - j0 * (j0 + 1.0));
}

// Reciprocal nudged upwards so that floor(a * r) == a / s exactly for integers
// a < 2^47, s >= 1: the product never falls below the true quotient and
// overshoots it by less than 1/s.  `approx` may be off by a few ulp.
__device__ inline double recip_up(double approx) { return approx * (1.0 + 0x1p-48); }
__device__ inline uint32_t floor_div(uint32_t a, double r_up) { return (uint32_t)((double)a * r_up); }

// 1/x to about an ulp: hardware seed plus two Newton steps (x > 0, normal).
__device__ inline double fast_recip(double x) {
    double r = __builtin_amdgcn_rcp(x);
    r = fma(fma(-x, r, 1.0), r, r);
    r = fma(fma(-x, r, 1.0), r, r);
    return r;
}

// sum_{j=1}^{n} max(alpha c_j, beta c_j + gamma) over contexts c_j = s + u j
// (r_u ~ 1/u): both sides are linear in c, so the series splits at one
// crossover; a step that lands within rounding of the crossover has equal
// sides, so an off-by-one there does not change the sum beyond an ulp.
template <bool ADDITIVE>
__device__ inline double attention_series(double alpha, double beta, double gamma, double s, double u, double r_u,
                                          double n) {
    const double tri = 0.5 * n * (n + 1.0);
    const double all = fma(u, tri, n * s);               // sum of c_j
    if (ADDITIVE) return fma(alpha + beta, all, n * gamma);
    if (alpha <= beta) return fma(beta, all, n * gamma); // bandwidth bound at every context
    double jm = floor((gamma * fast_recip(alpha - beta) - s) * r_u);
    jm = fmin(fmax(jm, 0.0), n);
    const double low = fma(u, 0.5 * jm * (jm + 1.0), jm * s);
    return fma(beta, low, fma(jm, gamma, alpha * (all - low)));
}

// Decode: steps j = 1..n with b tokens at context s + j.  Everything but
// attention is the same every step; attention is max(alpha ctx, beta ctx + gamma)
// with both sides linear in ctx, so the series splits at one crossover.
template <bool ADDITIVE>
__device__ inline double decode_time(const TimeCoef &t, uint32_t b_, uint32_t s_, uint32_t n_) {
    if (n_ == 0) return 0.0;
    const double b = (double)b_, s = (double)s_, n = (double)n_;
    const double base = fma(t.L, layer_base<ADDITIVE>(t, b), lm_head<ADDITIVE>(t, b));
    const double alpha = b * t.c_att, beta = b * t.m_att_k, gamma = b * t.m_att_t;
    double att;
    if (ADDITIVE) {
        att = (alpha + beta) * ctx_sum(s, 0.0, n) + n * gamma;
    } else if (alpha <= beta) {
        att = beta * ctx_sum(s, 0.0, n) + n * gamma;         // bandwidth bound at every context
    } else {
        // bandwidth bound while ctx <= gamma / (alpha - beta)
        double jm = floor(gamma / (alpha - beta) - s);
        jm = fmin(fmax(jm, 0.0), n);
        att = beta * ctx_sum(s, 0.0, jm) + jm * gamma + alpha * ctx_sum(s, jm, n);
    }
    return fma(n, base, t.L * att);
}

// Same prefill with the segment loop of long prompts summed in closed form and
// the integer divisions replaced by nudged reciprocals (r_s ~ 1/s, r_mbt ~ 1/mbt,
// both from recip_up).
template <bool ADDITIVE>
__device__ inline double prefill_time_fast(const TimeCoef &t, uint32_t b, uint32_t s, uint32_t mbt, double r_s,
                                           double r_mbt) {
    const double S = (double)s;
    if (s <= mbt) {
        uint32_t r = floor_div(mbt, r_s);
        r = r < b ? r : b;
        const uint32_t n_full = r == b ? 1u : floor_div(b, recip_up(fast_recip((double)r)));
        const uint32_t rem = b - n_full * r;
        double R = (double)r;
        double total = (double)n_full * pass_time<ADDITIVE>(t, R * S, R * S * S, R * S, R);
        if (rem > 0) {
            R = (double)rem;
            total += pass_time<ADDITIVE>(t, R * S, R * S * S, R * S, R);
        }
        return total;
    }
    // n_fs full segments of mbt tokens at contexts mbt, 2 mbt, ..; then the rest with the LM head
    const uint32_t n_seg = floor_div(s + mbt - 1, r_mbt);
    const double M = (double)mbt, n_fs = (double)(n_seg - 1);
    const double c_last = S - n_fs * M;
    const double att = attention_series<ADDITIVE>(M * t.c_att, t.m_att_k, M * t.m_att_t, 0.0, M, r_mbt, n_fs);
    const double one = fma(t.L, fma(n_fs, layer_base<ADDITIVE>(t, M), att), pass_time<ADDITIVE>(t, c_last, c_last * S, S, 1.0));
    return (double)b * one;
}

// The sample-independent part of a prefill: how the batch splits into passes.
struct PrefillPlan {
    bool segmented;      // prompt longer than the budget
    double n_full, R, rem, S;          // sub-batches: n_full passes of R prompts, then one of rem (0 = none)
    double n_fs, M, c_last, r_mbt;     // segments: n_fs full ones of M tokens, then c_last tokens with the LM head
};
__device__ inline PrefillPlan make_prefill_plan(uint32_t b, uint32_t s, uint32_t mbt, double r_s, double r_mbt) {
    PrefillPlan p;
    p.S = (double)s;
    p.segmented = s > mbt;
    p.n_full = p.R = p.rem = p.n_fs = p.c_last = 0.0;
    p.M = (double)mbt;
    p.r_mbt = r_mbt;
    if (!p.segmented) {
        uint32_t r = floor_div(mbt, r_s);
        r = r < b ? r : b;
        const uint32_t n_full = r == b ? 1u : floor_div(b, recip_up(fast_recip((double)r)));
        p.n_full = (double)n_full;
        p.R = (double)r;
        p.rem = (double)(b - n_full * r);
    } else {
        const uint32_t n_seg = floor_div(s + mbt - 1, r_mbt);
        p.n_fs = (double)(n_seg - 1);
        p.c_last = p.S - p.n_fs * p.M;
    }
    return p;
}
template <bool ADDITIVE>
__device__ inline double prefill_time_plan(const TimeCoef &t, const PrefillPlan &p, uint32_t b) {
    if (!p.segmented) {
        double total = p.n_full * pass_time<ADDITIVE>(t, p.R * p.S, p.R * p.S * p.S, p.R * p.S, p.R);
        if (p.rem > 0.0) total += pass_time<ADDITIVE>(t, p.rem * p.S, p.rem * p.S * p.S, p.rem * p.S, p.rem);
        return total;
    }
    const double att = attention_series<ADDITIVE>(p.M * t.c_att, t.m_att_k, p.M * t.m_att_t, 0.0, p.M, p.r_mbt, p.n_fs);
    const double one = fma(t.L, fma(p.n_fs, layer_base<ADDITIVE>(t, p.M), att),
                           pass_time<ADDITIVE>(t, p.c_last, p.c_last * p.S, p.S, 1.0));
    return (double)b * one;
}

template <bool ADDITIVE>
__device__ inline double decode_time_fast(const TimeCoef &t, uint32_t b_, uint32_t s_, uint32_t n_) {
    if (n_ == 0) return 0.0;
    const double b = (double)b_, n = (double)n_;
    const double base = fma(t.L, layer_base<ADDITIVE>(t, b), lm_head<ADDITIVE>(t, b));
    const double att = attention_series<ADDITIVE>(b * t.c_att, b * t.m_att_k, b * t.m_att_t, (double)s_, 1.0, 1.0, n);
    return fma(n, base, t.L * att);
}

struct MemResult {
    uint32_t b_max;
    bool feasible;
};

// available = capacity - weights / p; KV per request over block-rounded s_in + s_out.
__device__ inline MemResult memory_check(const Coef &c, double cap, uint32_t b, uint32_t s_in, uint32_t s_out,
                                         uint32_t blk) {
    MemResult r;
    const double c_avail = cap - c.w_gpu;
    const uint32_t tok = s_in + s_out;
    const uint32_t tok_req = (tok + blk - 1) / blk * blk;
    const double kv_req = (double)tok_req * c.kv_tok;
    if (c_avail > 0.0) {
        r.feasible = (double)b * kv_req <= c_avail;
        const double q = floor(c_avail / kv_req);
        r.b_max = q >= 4294967295.0 ? 4294967295u : (uint32_t)q;
    } else {
        r.feasible = false;
        r.b_max = 0u;
    }
    return r;
}

struct Knobs {
    uint32_t b, s_in, s_out, p, wbits, blk, mbt;
};

struct EvalResult {
    double t_prefill, t_decode;
};

template <bool ADDITIVE>
__device__ inline EvalResult evaluate_times(const TimeCoef &t, const Knobs &kn) {
    EvalResult r;
    r.t_prefill = prefill_time<ADDITIVE>(t, kn.b, kn.s_in, kn.mbt);
    r.t_decode = decode_time<ADDITIVE>(t, kn.b, kn.s_in, kn.s_out - 1);
    return r;
}

}  // namespace guide
