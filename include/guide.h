/*
 * guide.h -- C ABI of libguide: batched evaluation of GUIDE's LLM-inference
 * performance model over a space of deployment configurations on one AMD GPU,
 * step-level serving simulation, and constrained best-config / Pareto
 * selection (arXiv 2412.04788).
 *
 * Conventions for every entry point
 *   - Returns GUIDE_OK (0) or a negative guide_status; never throws or aborts.
 *     On a non-zero return nothing was enqueued and guide_last_error() holds a
 *     message.
 *   - Pointers marked HOST are read before the call returns and may be freed
 *     afterwards.  Pointers marked DEVICE are caller-owned device memory on the
 *     context's GPU (for instance torch tensors' data_ptr()); the library never
 *     frees or reallocates them.
 *   - Kernels are enqueued on `stream` (a hipStream_t passed as void*, NULL =
 *     the default stream).  The call returns after enqueueing; outputs are
 *     valid once the caller has synchronised the stream.  A launch failure is
 *     returned as GUIDE_E_DEVICE.
 *   - A context owns small device tables and scratch that its calls share.  A
 *     call on another stream than the context's previous call first makes its
 *     stream wait for the previous stream's work (an event, no host wait), so
 *     calls on one context never overlap on the GPU; use one context per stream
 *     for concurrency.  guide_select_static shares one scratch per GPU between
 *     all contexts (see there).
 *   - The first call on a stream after guide_create, or after the models,
 *     hardware, grid axes or efficiency samples changed, copies tables to the
 *     device (a pinned staging slot, a host wait on that slot's last use): such
 *     a call cannot be captured into a HIP graph.  Repeated calls with unchanged
 *     tables only launch kernels and can be captured.
 *   - Output capacity: a Pareto selection writes at most `capacity` indices and
 *     always reports the full front size in count[0]; a front larger than the
 *     capacity is not an error, the caller compares the two.
 *
 * Performance model (the reading of the paper implemented here)
 *   One forward pass over T tokens with attention workload Q (query x context
 *   pairs), K cached tokens read and n_lm LM-head rows costs, on one GPU of a
 *   tensor-parallel group of p,
 *       t_pass = L * (sum over layer ops of t_op + 2 * t_allreduce(T)) + t_lmhead
 *   where every op (Task: compute load F, data size B -- Parallel Simulator,
 *   "Task and GPU Models") takes t_op = max(F / peak, B / bandwidth) (Roofline
 *   Model for Performance Analysis) or F / peak + B / bandwidth under
 *   GUIDE_TIME_ADDITIVE (Time Calculation), and the all-reduce is the transfer
 *   term: 2(p-1)/p * bytes / link_bw + 2(p-1) * link_lat.
 *   Tasks of one layer (d_h = d / n_h, dq = n_h d_h, dkv = n_kv d_h, w = wbits / 8
 *   bytes per weight, activations and cached K/V 2 bytes per element, g_kv =
 *   ceil(n_kv / p) d_h, E_ld = min(E, k T) experts whose weights are read):
 *     qkv        F = 2 T d (dq + 2 dkv) / p     B = w d (dq + 2 dkv) / p + 2 T d + 2 T (dq + 2 dkv) / p
 *     attention  F = 4 dq Q / p                 B = 4 T dq / p + 4 g_kv K
 *     out-proj   F = 2 T dq d / p               B = w dq d / p + 2 T dq / p + 2 T d
 *     ffn-up     F = 2 T k (2 d d_ff) / p       B = w E_ld (2 d d_ff) / p + 2 T d + 4 T k d_ff / p
 *     ffn-down   F = 2 T k (d_ff d) / p         B = w E_ld (d_ff d) / p + 2 T k d_ff / p + 2 T d
 *     router     F = 2 T d E                    B = w d E + 2 T d + 2 T E        (only when E > 1)
 *     norms      F = 0                          B = 8 T d
 *   and once per pass the LM head over n_lm rows: F = 2 n_lm d V / p,
 *   B = w d V / p + 2 n_lm d + 2 n_lm V / p.  Stored parameters: L (2 d dq + 2 d dkv +
 *   3 E d d_ff + [E > 1] d E) + 2 V d; weights per GPU = w * parameters / p.
 *   Prefill of a static batch runs in sub-batches of floor(mbt / s_in) requests,
 *   or, for prompts longer than mbt, in ceil(s_in / mbt) segments per request
 *   (Model Analyzer, Dynamic Batch Size / Sequence Length Adjustment).  Decode
 *   runs s_out - 1 single-token passes with growing context.  TTFT is the
 *   prefill time; decode throughput is b * (s_out - 1) / t_decode = b / TPOT
 *   (Inference Engine, Step 2).  Memory: available = capacity - weights / p,
 *   KV per request = 2 * L * kv-width * block-rounded (s_in + s_out) * 2 bytes,
 *   B_max = floor(available / KV per request) (Inference Engine, Step 1).
 */
#ifndef GUIDE_H
#define GUIDE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct guide_ctx guide_ctx;

typedef enum {
    GUIDE_OK = 0,
    GUIDE_E_ARG = -1,      /* NULL required pointer, zero count, unknown enum            */
    GUIDE_E_RANGE = -2,    /* index range outside the grid, size beyond a stated limit    */
    GUIDE_E_NOMEM = -3,    /* workspace too small / allocation failed                     */
    GUIDE_E_DEVICE = -4    /* HIP runtime error, or not a gfx950 GPU                      */
} guide_status;

enum { GUIDE_TIME_ROOFLINE = 0, GUIDE_TIME_ADDITIVE = 1 };
enum { GUIDE_AXIS_GEOM2 = 0, GUIDE_AXIS_TABLE = 1 };
enum { GUIDE_SELECT_TOPK = 0, GUIDE_SELECT_PARETO = 1 };
enum { GUIDE_SIM_OK = 0, GUIDE_SIM_INFEASIBLE = 1, GUIDE_SIM_BAD_INPUT = 2, GUIDE_SIM_INTERNAL = 3 };
enum { GUIDE_SCHED_SPLIT_FUSE = 0, GUIDE_SCHED_PREFILL_FIRST = 1 };
enum { GUIDE_SIM_CLOSED_FORM_RUNS = 256 };   /* OR-ed into guide_simulate's scheduler argument */

#define GUIDE_MAX_MODELS 8
#define GUIDE_MAX_HW 64
#define GUIDE_MAX_AXIS_VALUES 64
#define GUIDE_MAX_EFF 64
#define GUIDE_MAX_CONSTRAINTS 4
#define GUIDE_MAX_GROUPS 64
#define GUIDE_MAX_TOPK 8
#define GUIDE_MAX_REQUESTS 1024
#define GUIDE_MAX_BUCKET_EDGES 15
#define GUIDE_HIST_BINS 256
#define GUIDE_LATTICE 1024
#define GUIDE_NO_INDEX UINT64_MAX
#define GUIDE_SELECT_MAX_ROWS 0xFFFFF000ull     /* guide_select: at most 2^32 - 4096 rows */

/* Decoder architecture.  E = k = 1 for a dense model; E experts with k active
 * per token otherwise.  n_h must divide d. */
typedef struct { uint32_t L, d, n_h, n_kv, d_ff, V, E, k; } guide_model;

/* Registered GPU (GPU model: compute performance, memory bandwidth,
 * communication bandwidth, latency) plus its memory capacity.  SI units. */
typedef struct { double peak_flops, hbm_bw, cap_bytes, link_bw, link_lat; } guide_hw;

/* One axis of the configuration grid.  GEOM2: value i = start << i (values
 * ignored).  TABLE: value i = values[i] (HOST, count entries).  count in
 * 1..GUIDE_MAX_AXIS_VALUES; every value must fit 32 bits.  The model and hw
 * axes hold indices into the tables given to guide_set_models / _hardware. */
typedef struct { uint32_t count, kind; uint64_t start; const uint64_t *values; } guide_axis;

/* Mixed-radix space, slowest axis first: flat index =
 * ((((((((m*N_hw+h)*N_b+ib)*N_in+iin)*N_out+iout)*N_tp+itp)*N_w+iw)*N_blk+iblk)*N_mbt+imbt.
 * wbits = weight bits per parameter (16, 8, 4); kv_block = tokens per KV block;
 * mbt = max batched tokens per pass.  Total size must be < 2^32; s_in and s_out
 * values must be < 2^31 and the largest s_in + s_out + kv_block < 2^32
 * (GUIDE_E_RANGE otherwise). */
typedef struct { guide_axis model, hw, batch, s_in, s_out, tp, wbits, kv_block, mbt; } guide_grid;

/* Multiplicative efficiency samples (HOST): peak *= e_c[i], bandwidth *= e_b[i].
 * n = 0 (or a NULL guide_eff) means the single nominal sample (1, 1). */
typedef struct { uint32_t n; const double *e_c; const double *e_b; } guide_eff;

/* Per-configuration outputs (DEVICE, each >= count elements; a NULL column is
 * not written).  Times in seconds; cost in GPU-hours per million generated
 * tokens; feasible = 1 iff available memory > 0 and b * KV-per-request fits
 * (inclusive); metrics are computed at the nominal batch even when infeasible. */
typedef struct {
    double *t_prefill, *t_decode, *t_batch, *decode_tok_s, *cost;
    uint32_t *b_max;
    uint8_t *feasible;
} guide_metrics;

/* Outputs of an efficiency sweep (eff.n > 1): mean (index-order sum / n) and
 * nearest-rank p10 / p90 (sorted[ceil(q n) - 1]) of TTFT and batch latency over
 * the samples; cost from the mean batch latency. */
typedef struct {
    double *ttft_mean, *ttft_p10, *ttft_p90, *t_batch_mean, *t_batch_p10, *t_batch_p90, *cost;
    uint32_t *b_max;
    uint8_t *feasible;
} guide_stats;

int guide_create(guide_ctx **ctx, int device);
void guide_destroy(guide_ctx *ctx);
const char *guide_last_error(const guide_ctx *ctx); /* ctx-owned, valid until the next call */

/* Copy n architectures / GPU records (HOST) into the context (synchronous). */
int guide_set_models(guide_ctx *ctx, const guide_model *models, uint32_t n);
int guide_set_hardware(guide_ctx *ctx, const guide_hw *hw, uint32_t n);

/*
 * Evaluate configurations [first, first + count) of `grid` (Parallel Simulator,
 * "Simulating Hybrid Parallelism": every generated configuration is simulated).
 * eff == NULL or eff->n <= 1: one sample, results to `out` (required).
 * eff->n in 2..GUIDE_MAX_EFF: sweep, results to `stats` (required; `out` ignored).
 * count == 0 is a no-op.  GUIDE_E_RANGE if first + count exceeds the grid.
 */
int guide_eval_grid(guide_ctx *ctx, const guide_grid *grid, uint64_t first, uint64_t count,
                    const guide_eff *eff, uint32_t time_model,
                    const guide_metrics *out, const guide_stats *stats, void *stream);

/*
 * Cluster-level columns for configurations [first, first + count) under a budget
 * of n_gpus identical GPUs (DEVICE, count elements each, NULL = skip):
 *   s_max            longest sequence that fits the batch: floor(available /
 *                    (b * KV bytes per token)), the paper's S_max = floor(C_available
 *                    / (2 N H B kv)) (Dynamic Sequence Length Adjustment); 0 when
 *                    the weights do not fit; saturates at UINT32_MAX;
 *   dp_max           data-parallel replicas: floor(n_gpus / tp);
 *   max_parallelism  dp_max * b_max (Inference Engine Step 1: Maximum Parallelism =
 *                    DP x available memory / kv per request);
 *   cluster_tok_s    dp_max * decode throughput (replicas are independent);
 *   paper_tok_s      the paper's multi-GPU throughput N * T_single / (1 + log2 P_TP)
 *                    with N = dp_max * tp GPUs in use, P_TP = tp and T_single the
 *                    decode throughput of the same configuration at tp = 1;
 *   b_adj            the adjusted batch B = min(B_input, B_max) (Dynamic Batch Size
 *                    Adjustment);
 *   n_sub_batches    prefill passes the batch is split into: ceil(b / split_size) with
 *                    split_size = min(b, floor(mbt / s_in)) prompts per pass, the
 *                    remainder forming one more pass; b when a prompt exceeds mbt (every
 *                    request then runs alone, in segments);
 *   n_segments       ceil(s_in / mbt): the splits of a long prompt (Dynamic Sequence
 *                    Length Adjustment: input length over split size, rounded up);
 *   s_adj            the adjusted sequence length min(s_in + s_out, s_max).
 * The metrics of guide_eval_grid are computed at the nominal batch and lengths;
 * these columns say what the adjustments would make of them.
 *
 * KV-cache reduction (Inference Engine Step 1: the memory analysis takes into
 * account "user inputs for optimization such as FlashAttention and H2O which
 * reduce the memory consumption"; the paper gives no formula).  Reading: the user
 * states kv_keep, the fraction of a request's KV entries that the reduction keeps
 * (H2O's heavy-hitter budget), 0 < kv_keep <= 1; 0 stands for 1.  A request then
 * holds ceil(kv_keep * (s_in + s_out)) entries (product in fp64), in whole blocks:
 *   b_max_kept       floor(available / KV bytes of that many entries), as b_max;
 *   feasible_kept    != 0 when the weights fit and the batch's kept entries fit;
 *   s_max_kept       floor(s_max / kv_keep) (division in fp64): the longest
 *                    sequence whose kept entries fit the batch; saturates.
 * FlashAttention lowers activation memory, which this analysis (weights + KV
 * cache) does not count: it has no column.  Other values of kv_keep (negative,
 * above 1, NaN): GUIDE_E_ARG.
 */
typedef struct {
    uint32_t *s_max, *dp_max;
    uint64_t *max_parallelism;
    double *cluster_tok_s, *paper_tok_s;
    uint32_t *b_adj, *n_sub_batches, *n_segments, *s_adj;
    double kv_keep;                             /* INPUT, by value */
    uint32_t *b_max_kept, *s_max_kept;
    uint8_t *feasible_kept;
} guide_extras;

int guide_eval_extras(guide_ctx *ctx, const guide_grid *grid, uint64_t first, uint64_t count, uint32_t n_gpus,
                      uint32_t time_model, const guide_extras *out, void *stream);

/*
 * Random-sampled space.  Candidate i draws fourteen 16-bit fields from one
 * Philox4x64-10 block (counter (i,0,0,0), key (seed,0)); field u picks entry
 * (u * n) >> 16 of an n-entry table.  All table pointers are HOST; the three
 * 1024-point lattices and `heads` have GUIDE_LATTICE entries, cap 6, tp 4,
 * wbits 3, kv_block 2, mbt 3, kv_choices 4 (0 = as many KV heads as heads).
 * hidden = 128 * heads; d_ff = 128 * floor(ratio * heads + 1/2) with
 * ratio = (ffn_lo_x2 + ffn_span_x2 * u / 65536) / 2; E = k = 1.
 */
typedef struct {
    const uint32_t *heads;
    const double *peak, *bw, *cap;
    const uint32_t *batch, *s_in, *s_out, *tp, *wbits, *kv_block, *mbt, *kv_choices;
    uint32_t layers_lo, layers_n, ffn_lo_x2, ffn_span_x2, vocab;
    double link_div; /* link_bw = bw / link_div, link_lat = 0 */
} guide_space;

/* Reduced outputs (DEVICE): feasible_count[1]; win_val / win_idx[n_edges + 1]:
 * per model-size bucket (number of edges <= stored parameters) the lowest cost
 * among feasible candidates with TTFT <= ttft_cap, lowest index on ties,
 * (+inf, GUIDE_NO_INDEX) when none; hist[GUIDE_HIST_BINS]: batch latency of
 * feasible candidates, 8 bins per octave over [2^-12, 2^20) s taken from the
 * fp64 bit pattern, clamped.  The library overwrites (does not accumulate).
 * Optional per-candidate columns (DEVICE, count elements, NULL = skip). */
typedef struct {
    uint64_t *feasible_count;
    double *win_val;
    uint64_t *win_idx;
    uint64_t *hist;
    double *t_prefill, *t_batch, *cost;
    uint32_t *b_max;
    uint8_t *feasible;
    uint32_t *bucket;
} guide_sampled_out;

int guide_eval_sampled(guide_ctx *ctx, const guide_space *space, uint64_t seed, uint64_t first, uint64_t count,
                       const double *bucket_edges /* HOST, ascending */, uint32_t n_edges, double ttft_cap,
                       uint32_t time_model, const guide_sampled_out *out, void *stream);

/*
 * Step-level continuous-batching simulation ("dynamic batch processing and
 * dynamic split flow", Overview) of n_cfg serving configurations.  Config c is
 * grid index cfg_idx[c] (DEVICE u32): its model, hardware, tp, wbits, kv_block
 * and mbt apply, its batch value is the cap on concurrent sequences, its
 * s_in / s_out digits are ignored.  Requests arrive at arrival_unit[i] / rate[c]
 * (rate DEVICE f64) with n_in[i] prompt and n_out[i] generated tokens (trace
 * HOST, n <= GUIDE_MAX_REQUESTS, arrivals non-decreasing, n_in, n_out >= 1).
 * Each loop: jump to the next arrival if idle; admit FCFS while arrived, under
 * the sequence cap and with ceil((in+out)/kv_block) free KV blocks (reserved
 * for the request's lifetime; stop at the first that cannot enter); run one
 * pass; advance time by t_pass.  The pass depends on `scheduler`, the two
 * framework behaviours the paper models (Inference Engine, Step 2):
 *   GUIDE_SCHED_SPLIT_FUSE    one decode token for every prefilled request +
 *                             prompt chunks in admission order under the
 *                             remaining mbt budget (dynamic split flow);
 *   GUIDE_SCHED_PREFILL_FIRST while admitted prompts wait: whole prompts only,
 *                             in admission order, as many as fit mbt (the first
 *                             always, even if longer), decoders pause; otherwise
 *                             one decode token for every running request
 *                             (dynamic batching without chunking).
 * With GUIDE_SIM_CLOSED_FORM_RUNS OR-ed into `scheduler`, a run of decode-only
 * passes (every running request decoding, none waiting for prompt chunks) is
 * not stepped: until the first decoder emits its last token or a request that
 * could be admitted has arrived, every pass has the same tokens and a context
 * that grows by one per decoder, so the r passes the stepped loop would run
 * (r = passes before the one that retires a decoder, or the least r whose
 * starting time now + time(r passes) has reached that arrival) are advanced at
 * once with time(r) = r * (pass without attention) + L * (the attention series
 * in closed form, split where attention turns from read bound to compute
 * bound).  Engine steps and request-steps count the same passes; times differ
 * from the stepped simulation by rounding only, so a result can differ from it
 * only where an admission test "arrived by now?" is decided within rounding.
 * Outputs (DEVICE, n_cfg each): nearest-rank p50 / p99 of TTFT, mean TPOT over
 * requests with n_out > 1, generated tokens / (last finish - first arrival),
 * status (GUIDE_SIM_INFEASIBLE when weights or one request do not fit,
 * GUIDE_SIM_BAD_INPUT for an index outside the grid or a rate <= 0: times +inf,
 * tokens_s 0), engine steps, and request-steps (sum over steps of decode
 * tokens + prompt chunks scheduled).
 * workspace: DEVICE, guide_simulate_workspace_bytes(n_cfg, n) bytes.
 */
typedef struct { uint32_t n; const double *arrival_unit; const uint32_t *n_in; const uint32_t *n_out; } guide_trace;
typedef struct {
    double *ttft_p50, *ttft_p99, *mean_tpot, *tokens_s;
    uint32_t *status;
    uint64_t *n_steps, *n_request_steps;
} guide_sim_out;

size_t guide_simulate_workspace_bytes(uint32_t n_cfg, uint32_t n_requests);
int guide_simulate(guide_ctx *ctx, const guide_grid *grid, const uint32_t *cfg_idx, const double *rate,
                   uint32_t n_cfg, const guide_trace *trace, uint32_t time_model, uint32_t scheduler,
                   const guide_sim_out *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Selection over n rows of DEVICE columns (the engine keeps the configurations
 * with the lowest inference time / highest throughput, top three -- Inference
 * Engine Step 2; Simulating Hybrid Parallelism).  A row passes when
 * feasible[row] != 0 (NULL = all), every constraint column[row] <= cap, and the
 * objective(s) are not NaN.
 * TOPK: per group g < n_groups (group NULL = one group; rows with group id >=
 *   n_groups are ignored) the first k passing rows in (objective ascending,
 *   row ascending) order -> idx[g*k + j], val[g*k + j] ((GUIDE_NO_INDEX, +inf)
 *   when fewer pass); count[g] = passing rows.  k <= GUIDE_MAX_TOPK,
 *   n_groups <= GUIDE_MAX_GROUPS.
 * PARETO: rows not dominated in (objective, objective_y), both minimised (row
 *   j dominates i when x_j <= x_i, y_j <= y_i and one is strict; equal rows are
 *   all kept) -> idx[0 .. min(front, capacity)) sorted by (x, y, row);
 *   count[0] = front size, which may exceed capacity (the caller compares);
 *   val unused.
 * workspace: DEVICE, guide_select_workspace_bytes(spec, n) bytes.
 */
typedef struct { const double *column; double cap; } guide_constraint;
typedef struct {
    uint32_t mode;
    const double *objective;
    const double *objective_y;
    const uint8_t *feasible;
    uint32_t n_constraints;
    guide_constraint constraints[GUIDE_MAX_CONSTRAINTS];
    const uint32_t *group;
    uint32_t n_groups;
    uint32_t k;
} guide_select_spec;
typedef struct { uint64_t *idx; double *val; uint64_t *count; uint64_t capacity; } guide_select_out;

size_t guide_select_workspace_bytes(const guide_select_spec *spec, uint64_t n);
int guide_select(guide_ctx *ctx, const guide_select_spec *spec, uint64_t n, const guide_select_out *out,
                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * guide_select for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  The same selection and the same outputs as guide_select; the
 * workspace and the Pareto tables live in one static device array inside the
 * library (about 60 MiB on every GPU the library runs on, held until the
 * process ends; its address is taken once per device in guide_create).  The
 * call allocates and frees nothing.  Limits: the selection's workspace
 * (guide_select_workspace_bytes) must fit the array, which holds a Pareto
 * selection over GUIDE_STATIC_SELECT_MAX_ROWS rows and a top-k selection of
 * any size; beyond that GUIDE_E_RANGE is returned and nothing is enqueued.
 * Every call on one GPU, from any context, uses that GPU's one array: the kernels
 * of a call rewrite every part of it before reading it, so it needs no clearing
 * between calls and keeps nothing from the last one, but two calls that overlap
 * on one GPU (different streams, different contexts) race.
 */
#define GUIDE_STATIC_SELECT_MAX_ROWS (1ull << 21)
int guide_select_static(guide_ctx *ctx, const guide_select_spec *spec, uint64_t n, const guide_select_out *out,
                        void *stream);

/*
 * Evaluate and select in one call: the same results as guide_eval_grid(out) with
 * one efficiency sample followed by guide_select for each of the n_sel
 * selections on the columns of `out` (rows = the `count` evaluated
 * configurations, one group) -- the engine's "evaluate every configuration, keep
 * the best" (Inference Engine Step 2; Simulating Hybrid Parallelism) -- in fewer
 * launches: with a top-k and a Pareto selection, the small kernels of one ride
 * along with the large kernels of the other, and a top-k (k <= 4) that refers only
 * to the Pareto selection's two columns has no pass of its own.  Columns are named
 * by GUIDE_COL_*; a tile kernel exists for up to four values on each of the two
 * fastest axes.
 * At most one selection per mode (n_sel <= 2; n_sel = 0 is a plain evaluation).
 * Every column that a selection refers to, and `feasible` when use_feasible is
 * set, must be present in `out` (GUIDE_E_ARG otherwise), with one exception: for
 * a grid whose two fastest axes have a tile kernel, a top-k selection with
 * k <= 4 whose columns are not all stored is reduced inside the evaluation
 * kernel instead, so the best configurations can be found without storing the
 * grid.
 * workspace: DEVICE, guide_eval_select_workspace_bytes(sel, n_sel, count) bytes.
 */
enum { GUIDE_COL_T_PREFILL = 0, GUIDE_COL_T_DECODE = 1, GUIDE_COL_T_BATCH = 2, GUIDE_COL_DECODE_TOK_S = 3,
       GUIDE_COL_COST = 4, GUIDE_NUM_COLS = 5 };
typedef struct { uint32_t column; uint32_t reserved; double cap; } guide_column_constraint;
typedef struct {
    uint32_t mode;          /* GUIDE_SELECT_TOPK | GUIDE_SELECT_PARETO */
    uint32_t objective;     /* GUIDE_COL_*, minimised */
    uint32_t objective_y;   /* Pareto only */
    uint32_t use_feasible;  /* != 0: rows with feasible == 0 do not pass */
    uint32_t n_constraints;
    uint32_t k;             /* top-k only, <= GUIDE_MAX_TOPK */
    guide_column_constraint constraints[GUIDE_MAX_CONSTRAINTS];
    guide_select_out out;   /* as for guide_select */
} guide_column_select;

size_t guide_eval_select_workspace_bytes(const guide_column_select *sel, uint32_t n_sel, uint64_t count);
int guide_eval_select(guide_ctx *ctx, const guide_grid *grid, uint64_t first, uint64_t count, const guide_eff *eff,
                      uint32_t time_model, const guide_metrics *out, const guide_column_select *sel, uint32_t n_sel,
                      void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* GUIDE_H */
