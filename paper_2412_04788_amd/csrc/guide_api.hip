// C ABI of libguide: argument validation, context tables, kernel launches.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "kernels.hpp"
#include "guide_diag.h"

using namespace guide;

struct guide_ctx {
    int device = 0;
    uint32_t n_models = 0, n_hw = 0;
    DevTables host_tab;              // staging copy of the device tables
    DevTables sent_tab;              // what dev_tab holds (valid when sent_valid), enqueued on sent_stream
    bool sent_valid = false;
    hipStream_t sent_stream = nullptr;
    DevTables *dev_tab = nullptr;
    uint64_t tab_gen = 0;            // counts uploads of dev_tab
    void *dev_tile = nullptr;        // tables derived from (grid description, dev_tab) for the tile kernels
    GridDesc tile_desc;              // what dev_tile was derived from: this description ...
    uint64_t tile_gen = 0;           // ... and this upload of dev_tab (0 = never)
    SpaceTables *dev_space = nullptr;
    TraceDev *dev_trace = nullptr;
    void *sampled_scratch = nullptr;
    void *select_scratch = nullptr;   // tables of the Pareto kernels, see select.hip
    // Ring of pinned staging slots for the small per-call tables: the async copy
    // reads the slot later, so a slot is reused only after its event has passed.
    static constexpr int kSlots = 4;
    static constexpr size_t kSlotBytes = sizeof(SpaceTables) > sizeof(TraceDev) ? sizeof(SpaceTables) : sizeof(TraceDev);
    void *slot[kSlots] = {nullptr, nullptr, nullptr, nullptr};
    hipEvent_t slot_ev[kSlots] = {nullptr, nullptr, nullptr, nullptr};
    int next_slot = 0;
    // kernel timing aid: event pairs around evaluation kernels (guide_profile_enable)
    std::vector<hipEvent_t> prof_ev;     // 2 * capacity events
    uint32_t prof_used = 0;              // timed launches since the last read
    uint32_t prof_every = 1, prof_seen = 0;   // every prof_every-th launch is timed
    hipStream_t prof_stream = nullptr;
    // the stream of the last enqueueing call, and the event that orders a call on another stream after it
    hipStream_t last_stream = nullptr;
    bool used = false;
    hipEvent_t order_ev = nullptr;
    char err[256] = {0};
};
static_assert(guide_ctx::kSlotBytes >= sizeof(DevTables), "staging slot too small");

// Device memory of guide_select_static, which may not allocate: the tables of the Pareto kernels
// (kSelectScratchMax bytes) followed by the selection workspace (kStaticWsBytes, enough for a Pareto
// selection over GUIDE_STATIC_SELECT_MAX_ROWS rows or any top-k selection).  Every GPU holds its own copy
// at its own address: host code never uses the array's name as a pointer, only the address that
// hipGetSymbolAddress returned for the device (static_scratch_of).
constexpr size_t kStaticWsBytes = (size_t)GUIDE_STATIC_SELECT_MAX_ROWS * 30 + 256;
static __device__ __align__(256) unsigned char scratch[kSelectScratchMax + kStaticWsBytes];
constexpr int kMaxDevices = 64;
static void *g_static_scratch[kMaxDevices];      // per device: address of `scratch` there, set by guide_create

namespace {

int fail(guide_ctx *ctx, int code, const char *fmt, ...) {
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof ctx->err, fmt, ap);
        va_end(ap);
    }
    return code;
}

int hip_fail(guide_ctx *ctx, hipError_t e, const char *what) {
    return fail(ctx, GUIDE_E_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

#define GUIDE_HIP(ctx, call)                                       \
    do {                                                           \
        hipError_t e_ = (call);                                    \
        if (e_ != hipSuccess) return hip_fail(ctx, e_, #call);     \
    } while (0)

struct DeviceGuard {
    int prev = -1;
    bool ok = false;
    explicit DeviceGuard(int dev) {
        if (hipGetDevice(&prev) == hipSuccess && (prev == dev || hipSetDevice(dev) == hipSuccess)) ok = true;
        if (prev == dev) prev = -1;
    }
    ~DeviceGuard() {
        if (prev >= 0) (void)hipSetDevice(prev);
    }
};

const guide_axis *axis_of(const guide_grid *g, int a) {
    const guide_axis *ax[kNumAxes] = {&g->model, &g->hw, &g->batch, &g->s_in, &g->s_out,
                                      &g->tp,    &g->wbits, &g->kv_block, &g->mbt};
    return ax[a];
}

const char *kAxisName[kNumAxes] = {"model", "hw", "batch", "s_in", "s_out", "tp", "wbits", "kv_block", "mbt"};

// Validates the grid, fills the staging tables and the launch descriptor.
int prepare_grid(guide_ctx *ctx, const guide_grid *grid, GridDesc *desc, uint64_t *size) {
    if (!grid) return fail(ctx, GUIDE_E_ARG, "grid is NULL");
    if (ctx->n_models == 0 || ctx->n_hw == 0)
        return fail(ctx, GUIDE_E_ARG, "guide_set_models and guide_set_hardware must be called first");
    uint64_t total = 1;
    for (int a = 0; a < kNumAxes; ++a) {
        const guide_axis *ax = axis_of(grid, a);
        if (ax->count == 0 || ax->count > GUIDE_MAX_AXIS_VALUES)
            return fail(ctx, GUIDE_E_ARG, "axis %s: count %u outside 1..%d", kAxisName[a], ax->count,
                        GUIDE_MAX_AXIS_VALUES);
        if (ax->kind != GUIDE_AXIS_GEOM2 && ax->kind != GUIDE_AXIS_TABLE)
            return fail(ctx, GUIDE_E_ARG, "axis %s: unknown kind %u", kAxisName[a], ax->kind);
        if (ax->kind == GUIDE_AXIS_TABLE && !ax->values)
            return fail(ctx, GUIDE_E_ARG, "axis %s: TABLE axis without values", kAxisName[a]);
        for (uint32_t i = 0; i < ax->count; ++i) {
            uint64_t v;
            if (ax->kind == GUIDE_AXIS_GEOM2) {
                if (i >= 32 || (ax->start << i) >> i != ax->start)
                    return fail(ctx, GUIDE_E_RANGE, "axis %s: start << %u overflows", kAxisName[a], i);
                v = ax->start << i;
            } else {
                v = ax->values[i];
            }
            if (v > 0xFFFFFFFFull) return fail(ctx, GUIDE_E_RANGE, "axis %s: value does not fit 32 bits", kAxisName[a]);
            if (a == AX_MODEL && v >= ctx->n_models)
                return fail(ctx, GUIDE_E_RANGE, "model axis: index %llu >= %u models", (unsigned long long)v, ctx->n_models);
            if (a == AX_HW && v >= ctx->n_hw)
                return fail(ctx, GUIDE_E_RANGE, "hw axis: index %llu >= %u records", (unsigned long long)v, ctx->n_hw);
            if (a >= AX_BATCH && v == 0) return fail(ctx, GUIDE_E_ARG, "axis %s: zero value", kAxisName[a]);
            if ((a == AX_SIN || a == AX_SOUT) && v > 0x7FFFFFFFull)
                return fail(ctx, GUIDE_E_RANGE, "axis %s: length above 2^31", kAxisName[a]);
            ctx->host_tab.axis_vals[a][i] = (uint32_t)v;
        }
        desc->div[a] = make_div32(ax->count);
        total *= ax->count;
        if (total >= (1ull << 32)) return fail(ctx, GUIDE_E_RANGE, "grid has 2^32 or more configurations");
    }
    // block rounding adds s_in + s_out + kv_block - 1 in 32 bits
    uint64_t longest = 0;
    for (int a : {AX_SIN, AX_SOUT, AX_BLK}) {
        uint32_t m = 0;
        for (uint32_t i = 0; i < axis_of(grid, a)->count; ++i) m = ctx->host_tab.axis_vals[a][i] > m ? ctx->host_tab.axis_vals[a][i] : m;
        longest += m;
    }
    if (longest >= (1ull << 32))
        return fail(ctx, GUIDE_E_RANGE, "largest s_in + s_out + kv_block is 2^32 or more");
    desc->n_models = ctx->n_models;
    desc->n_hw = ctx->n_hw;
    *size = total;
    return GUIDE_OK;
}

// Stream-ordered upload of a small host table through a pinned slot.
int stage_upload(guide_ctx *ctx, void *dst_dev, const void *src_host, size_t bytes, hipStream_t stream) {
    const int i = ctx->next_slot;
    ctx->next_slot = (i + 1) % guide_ctx::kSlots;
    GUIDE_HIP(ctx, hipEventSynchronize(ctx->slot_ev[i]));
    memcpy(ctx->slot[i], src_host, bytes);
    GUIDE_HIP(ctx, hipMemcpyAsync(dst_dev, ctx->slot[i], bytes, hipMemcpyHostToDevice, stream));
    GUIDE_HIP(ctx, hipEventRecord(ctx->slot_ev[i], stream));
    return GUIDE_OK;
}

// The grid tables rarely change between calls: skip the copy when the device
// already holds (or, in stream order, will hold) the same bytes.
int upload_tables(guide_ctx *ctx, hipStream_t stream) {
    if (ctx->sent_valid && ctx->sent_stream == stream && memcmp(&ctx->sent_tab, &ctx->host_tab, sizeof(DevTables)) == 0)
        return GUIDE_OK;
    ctx->sent_valid = false;
    const int rc = stage_upload(ctx, ctx->dev_tab, &ctx->host_tab, sizeof(DevTables), stream);
    if (rc) return rc;
    memcpy(&ctx->sent_tab, &ctx->host_tab, sizeof(DevTables));
    ctx->sent_valid = true;
    ctx->sent_stream = stream;
    ++ctx->tab_gen;
    return GUIDE_OK;
}

// upload_tables, then the derived tables of the tile kernels when the upload or the grid's radices
// are new (a new stream re-uploads, so the derivation is ordered on the stream that reads it).
int upload_grid_tables(guide_ctx *ctx, const GridDesc &desc, hipStream_t stream) {
    const int rc = upload_tables(ctx, stream);
    if (rc) return rc;
    if (ctx->tile_gen == ctx->tab_gen && memcmp(&ctx->tile_desc, &desc, sizeof desc) == 0) return GUIDE_OK;
    const hipError_t e = launch_tile_tables(desc, ctx->dev_tab, ctx->dev_tile, stream);
    if (e != hipSuccess) return hip_fail(ctx, e, "tile tables launch");
    memcpy(&ctx->tile_desc, &desc, sizeof desc);
    ctx->tile_gen = ctx->tab_gen;
    return GUIDE_OK;
}

// Calls on one context share its device tables and scratch.  A call that arrives on another stream than the
// previous one first makes its stream wait for everything enqueued on the previous stream (no host wait; nothing
// happens while the stream stays the same).
int order_after_previous(guide_ctx *ctx, hipStream_t stream) {
    if (ctx->used && stream != ctx->last_stream) {
        hipError_t e = hipEventRecord(ctx->order_ev, ctx->last_stream);
        if (e == hipSuccess) e = hipStreamWaitEvent(stream, ctx->order_ev, 0);
        if (e != hipSuccess) {                     // e.g. the previous stream no longer exists
            (void)hipGetLastError();
            e = hipDeviceSynchronize();
        }
        if (e != hipSuccess) return hip_fail(ctx, e, "ordering after the previous stream");
    }
    ctx->used = true;
    ctx->last_stream = stream;
    return GUIDE_OK;
}

bool time_model_ok(uint32_t tm) { return tm == GUIDE_TIME_ROOFLINE || tm == GUIDE_TIME_ADDITIVE; }

// The event pair for the next evaluation kernel, when timing is enabled, this launch's turn has come and
// a pair is left (empty otherwise); the launch attaches the events to the kernel's dispatch.
LaunchTiming next_timing(guide_ctx *ctx) {
    LaunchTiming t;
    if (ctx->prof_ev.empty()) return t;
    if (ctx->prof_seen++ % ctx->prof_every != 0 || 2 * (size_t)ctx->prof_used + 1 >= ctx->prof_ev.size()) return t;
    t.start = ctx->prof_ev[2 * ctx->prof_used];
    t.stop = ctx->prof_ev[2 * ctx->prof_used + 1];
    ++ctx->prof_used;
    return t;
}

// Two more pairs for the selection passes of a call whose evaluation kernel is timed (false: too few left).
bool pass_timing(guide_ctx *ctx, LaunchTiming (&t)[2]) {
    if (2 * ((size_t)ctx->prof_used + 2) > ctx->prof_ev.size()) return false;
    for (int i = 0; i < 2; ++i) {
        t[i].start = ctx->prof_ev[2 * ctx->prof_used];
        t[i].stop = ctx->prof_ev[2 * ctx->prof_used + 1];
        ++ctx->prof_used;
    }
    return true;
}

const double *metric_column(const guide_metrics &m, uint32_t id) {
    switch (id) {
        case GUIDE_COL_T_PREFILL: return m.t_prefill;
        case GUIDE_COL_T_DECODE: return m.t_decode;
        case GUIDE_COL_T_BATCH: return m.t_batch;
        case GUIDE_COL_DECODE_TOK_S: return m.decode_tok_s;
        case GUIDE_COL_COST: return m.cost;
        default: return nullptr;
    }
}

size_t round_up_256(size_t b) { return (b + 255) / 256 * 256; }

// guide_select's description of a column selection (column pointers from `out`; NULL where not stored).
guide_select_spec spec_of(const guide_column_select &c, const guide_metrics &out) {
    guide_select_spec s;
    memset(&s, 0, sizeof s);
    s.mode = c.mode;
    s.objective = metric_column(out, c.objective);
    s.objective_y = c.mode == GUIDE_SELECT_PARETO ? metric_column(out, c.objective_y) : nullptr;
    s.feasible = c.use_feasible ? out.feasible : nullptr;
    s.n_constraints = c.n_constraints;
    for (uint32_t i = 0; i < c.n_constraints && i < GUIDE_MAX_CONSTRAINTS; ++i) {
        s.constraints[i].column = metric_column(out, c.constraints[i].column);
        s.constraints[i].cap = c.constraints[i].cap;
    }
    s.group = nullptr;
    s.n_groups = 1;
    s.k = c.k;
    return s;
}

bool columns_present(const guide_column_select &c, const guide_metrics &out) {
    const guide_select_spec s = spec_of(c, out);
    if (!s.objective) return false;
    if (c.mode == GUIDE_SELECT_PARETO && !s.objective_y) return false;
    if (c.use_feasible && !out.feasible) return false;
    for (uint32_t i = 0; i < c.n_constraints; ++i)
        if (!s.constraints[i].column) return false;
    return true;
}

FusedFilter filter_of(const guide_column_select &c) {
    FusedFilter f;
    memset(&f, 0, sizeof f);
    f.use_feasible = c.use_feasible ? 1u : 0u;
    f.n_con = c.n_constraints;
    for (uint32_t i = 0; i < c.n_constraints; ++i) {
        f.col[i] = c.constraints[i].column;
        f.cap[i] = c.constraints[i].cap;
    }
    return f;
}

}  // namespace

extern "C" {

int guide_create(guide_ctx **out, int device) {
    if (!out) return GUIDE_E_ARG;
    *out = nullptr;
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess || device < 0 || device >= n_dev) return GUIDE_E_DEVICE;
    guide_ctx *ctx = new (std::nothrow) guide_ctx;
    if (!ctx) return GUIDE_E_NOMEM;
    ctx->device = device;
    memset(&ctx->host_tab, 0, sizeof ctx->host_tab);
    memset(&ctx->sent_tab, 0, sizeof ctx->sent_tab);
    memset(&ctx->tile_desc, 0, sizeof ctx->tile_desc);
    DeviceGuard guard(device);
    if (!guard.ok || hipMalloc((void **)&ctx->dev_tab, sizeof(DevTables)) != hipSuccess ||
        hipMalloc((void **)&ctx->dev_space, sizeof(SpaceTables)) != hipSuccess ||
        hipMalloc((void **)&ctx->dev_trace, sizeof(TraceDev)) != hipSuccess ||
        hipMalloc(&ctx->sampled_scratch, sampled_scratch_bytes()) != hipSuccess ||
        hipMalloc(&ctx->select_scratch, select_scratch_bytes()) != hipSuccess ||
        hipMalloc(&ctx->dev_tile, tile_tables_bytes()) != hipSuccess ||
        hipStreamSynchronize(nullptr) != hipSuccess) {
        guide_destroy(ctx);
        return GUIDE_E_DEVICE;
    }
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess || strncmp(prop.gcnArchName, "gfx950", 6) != 0 ||
        prop.multiProcessorCount <= 0 || hipEventCreateWithFlags(&ctx->order_ev, hipEventDisableTiming) != hipSuccess) {
        guide_destroy(ctx);                        // the kernels are built for gfx950 only
        return GUIDE_E_DEVICE;
    }
    // address of this device's copy of the static scratch (the device is current here)
    if (device < kMaxDevices && !g_static_scratch[device]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            guide_destroy(ctx);
            return GUIDE_E_DEVICE;
        }
        g_static_scratch[device] = p;
    }
    for (int i = 0; i < guide_ctx::kSlots; ++i) {
        if (hipHostMalloc(&ctx->slot[i], guide_ctx::kSlotBytes, hipHostMallocDefault) != hipSuccess ||
            hipEventCreateWithFlags(&ctx->slot_ev[i], hipEventDisableTiming) != hipSuccess) {
            guide_destroy(ctx);
            return GUIDE_E_DEVICE;
        }
    }
    *out = ctx;
    return GUIDE_OK;
}

void guide_destroy(guide_ctx *ctx) {
    if (!ctx) return;
    DeviceGuard guard(ctx->device);
    if (ctx->dev_tab) (void)hipFree(ctx->dev_tab);
    if (ctx->dev_space) (void)hipFree(ctx->dev_space);
    if (ctx->dev_trace) (void)hipFree(ctx->dev_trace);
    if (ctx->sampled_scratch) (void)hipFree(ctx->sampled_scratch);
    if (ctx->select_scratch) (void)hipFree(ctx->select_scratch);
    if (ctx->dev_tile) (void)hipFree(ctx->dev_tile);
    for (int i = 0; i < guide_ctx::kSlots; ++i) {
        if (ctx->slot_ev[i]) { (void)hipEventSynchronize(ctx->slot_ev[i]); (void)hipEventDestroy(ctx->slot_ev[i]); }
        if (ctx->slot[i]) (void)hipHostFree(ctx->slot[i]);
    }
    for (hipEvent_t e : ctx->prof_ev) (void)hipEventDestroy(e);
    if (ctx->order_ev) (void)hipEventDestroy(ctx->order_ev);
    delete ctx;
}

const char *guide_last_error(const guide_ctx *ctx) { return ctx ? ctx->err : "guide: NULL context"; }

int guide_set_models(guide_ctx *ctx, const guide_model *models, uint32_t n) {
    if (!ctx) return GUIDE_E_ARG;
    if (!models || n == 0 || n > GUIDE_MAX_MODELS) return fail(ctx, GUIDE_E_ARG, "models: need 1..%d rows", GUIDE_MAX_MODELS);
    for (uint32_t i = 0; i < n; ++i) {
        const guide_model &m = models[i];
        if (!m.L || !m.d || !m.n_h || !m.n_kv || !m.d_ff || !m.V || !m.E || !m.k)
            return fail(ctx, GUIDE_E_ARG, "model %u: zero field", i);
        if (m.d % m.n_h) return fail(ctx, GUIDE_E_ARG, "model %u: n_h does not divide d", i);
        if (m.k > m.E) return fail(ctx, GUIDE_E_ARG, "model %u: k > E", i);
    }
    memcpy(ctx->host_tab.models, models, sizeof(guide_model) * n);
    ctx->n_models = n;
    return GUIDE_OK;
}

int guide_set_hardware(guide_ctx *ctx, const guide_hw *hw, uint32_t n) {
    if (!ctx) return GUIDE_E_ARG;
    if (!hw || n == 0 || n > GUIDE_MAX_HW) return fail(ctx, GUIDE_E_ARG, "hardware: need 1..%d rows", GUIDE_MAX_HW);
    for (uint32_t i = 0; i < n; ++i) {
        const guide_hw &h = hw[i];
        if (!(h.peak_flops > 0.0) || !(h.hbm_bw > 0.0) || !(h.cap_bytes > 0.0) || !(h.link_bw > 0.0) ||
            !(h.link_lat >= 0.0))
            return fail(ctx, GUIDE_E_ARG, "hardware %u: non-positive field", i);
    }
    memcpy(ctx->host_tab.hw, hw, sizeof(guide_hw) * n);
    ctx->n_hw = n;
    return GUIDE_OK;
}

int guide_eval_grid(guide_ctx *ctx, const guide_grid *grid, uint64_t first, uint64_t count, const guide_eff *eff,
                    uint32_t time_model, const guide_metrics *out, const guide_stats *stats, void *stream_) {
    if (!ctx) return GUIDE_E_ARG;
    hipStream_t stream = (hipStream_t)stream_;
    if (!time_model_ok(time_model)) return fail(ctx, GUIDE_E_ARG, "unknown time model %u", time_model);
    GridDesc desc;
    uint64_t size = 0;
    int rc = prepare_grid(ctx, grid, &desc, &size);
    if (rc) return rc;
    if (first > size || count > size - first)
        return fail(ctx, GUIDE_E_RANGE, "range [%llu, +%llu) outside the grid of %llu", (unsigned long long)first,
                    (unsigned long long)count, (unsigned long long)size);
    const uint32_t n_eff = eff ? eff->n : 0;
    if (n_eff > GUIDE_MAX_EFF) return fail(ctx, GUIDE_E_RANGE, "more than %d efficiency samples", GUIDE_MAX_EFF);
    if (n_eff > 0 && (!eff->e_c || !eff->e_b)) return fail(ctx, GUIDE_E_ARG, "efficiency arrays are NULL");
    for (uint32_t i = 0; i < n_eff; ++i)
        if (!(eff->e_c[i] > 0.0) || !(eff->e_b[i] > 0.0) || std::isinf(eff->e_c[i]) || std::isinf(eff->e_b[i]))
            return fail(ctx, GUIDE_E_ARG, "efficiency sample %u is not a positive finite number", i);
    if (n_eff > 1 && !stats) return fail(ctx, GUIDE_E_ARG, "sweep needs a guide_stats");
    if (n_eff <= 1 && !out) return fail(ctx, GUIDE_E_ARG, "guide_metrics is NULL");
    if (count == 0) return GUIDE_OK;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return fail(ctx, GUIDE_E_DEVICE, "cannot select device %d", ctx->device);
    if (int rc_order = order_after_previous(ctx, stream)) return rc_order;
    for (uint32_t i = 0; i < n_eff; ++i) {
        ctx->host_tab.eff_c[i] = eff->e_c[i];
        ctx->host_tab.eff_b[i] = eff->e_b[i];
    }
    rc = n_eff > 1 ? upload_tables(ctx, stream) : upload_grid_tables(ctx, desc, stream);
    if (rc) return rc;
    hipError_t e;
    if (n_eff > 1) {
        e = launch_eval_sweep(desc, ctx->dev_tab, (uint32_t)first, (uint32_t)count, n_eff,
                              time_model == GUIDE_TIME_ADDITIVE, *stats, stream);
    } else {
        const double e_c = n_eff ? eff->e_c[0] : 1.0, e_b = n_eff ? eff->e_b[0] : 1.0;
        e = launch_eval_grid(desc, ctx->dev_tab, ctx->dev_tile, (uint32_t)first, (uint32_t)count, e_c, e_b,
                             time_model == GUIDE_TIME_ADDITIVE, *out, stream, next_timing(ctx));
    }
    if (e != hipSuccess) return hip_fail(ctx, e, "eval_grid launch");
    return GUIDE_OK;
}

size_t guide_eval_select_workspace_bytes(const guide_column_select *sel, uint32_t n_sel, uint64_t count) {
    if (!sel) return 0;
    size_t total = 0;
    for (uint32_t i = 0; i < n_sel; ++i) {
        guide_select_spec s;
        memset(&s, 0, sizeof s);
        s.mode = sel[i].mode;
        s.n_groups = 1;
        s.k = sel[i].k;
        size_t b = select_workspace_bytes(s, count);
        if (sel[i].mode == GUIDE_SELECT_TOPK && b < topk_partials_bytes()) b = topk_partials_bytes();
        total += round_up_256(b);
    }
    return total;
}

int guide_eval_select(guide_ctx *ctx, const guide_grid *grid, uint64_t first, uint64_t count, const guide_eff *eff,
                      uint32_t time_model, const guide_metrics *out, const guide_column_select *sel, uint32_t n_sel,
                      void *workspace, size_t workspace_bytes, void *stream_) {
    if (!ctx) return GUIDE_E_ARG;
    hipStream_t stream = (hipStream_t)stream_;
    if (!time_model_ok(time_model)) return fail(ctx, GUIDE_E_ARG, "unknown time model %u", time_model);
    if (!out) return fail(ctx, GUIDE_E_ARG, "guide_metrics is NULL");
    if (n_sel > 2 || (n_sel && !sel)) return fail(ctx, GUIDE_E_ARG, "at most two selections, one per mode");
    GridDesc desc;
    uint64_t size = 0;
    int rc = prepare_grid(ctx, grid, &desc, &size);
    if (rc) return rc;
    if (first > size || count > size - first)
        return fail(ctx, GUIDE_E_RANGE, "range [%llu, +%llu) outside the grid of %llu", (unsigned long long)first,
                    (unsigned long long)count, (unsigned long long)size);
    const uint32_t n_eff = eff ? eff->n : 0;
    if (n_eff > 1) return fail(ctx, GUIDE_E_ARG, "evaluate-and-select takes one efficiency sample");
    if (n_eff == 1 && (!eff->e_c || !eff->e_b)) return fail(ctx, GUIDE_E_ARG, "efficiency arrays are NULL");
    if (n_eff == 1 && (!(eff->e_c[0] > 0.0) || !(eff->e_b[0] > 0.0) || std::isinf(eff->e_c[0]) || std::isinf(eff->e_b[0])))
        return fail(ctx, GUIDE_E_ARG, "efficiency sample is not a positive finite number");
    const bool can_fuse = count > 0 && eval_grid_can_fuse(desc);
    const guide_column_select *topk = nullptr, *pareto = nullptr;
    bool topk_folded = false;
    for (uint32_t i = 0; i < n_sel; ++i) {
        const guide_column_select &c = sel[i];
        if (c.mode != GUIDE_SELECT_TOPK && c.mode != GUIDE_SELECT_PARETO)
            return fail(ctx, GUIDE_E_ARG, "selection %u: unknown mode %u", i, c.mode);
        if ((c.mode == GUIDE_SELECT_TOPK ? topk : pareto) != nullptr)
            return fail(ctx, GUIDE_E_ARG, "two selections of the same mode");
        if (c.objective >= GUIDE_NUM_COLS || (c.mode == GUIDE_SELECT_PARETO && c.objective_y >= GUIDE_NUM_COLS))
            return fail(ctx, GUIDE_E_ARG, "selection %u: unknown column", i);
        if (c.n_constraints > GUIDE_MAX_CONSTRAINTS)
            return fail(ctx, GUIDE_E_ARG, "selection %u: more than %d constraints", i, GUIDE_MAX_CONSTRAINTS);
        for (uint32_t k = 0; k < c.n_constraints; ++k)
            if (c.constraints[k].column >= GUIDE_NUM_COLS)
                return fail(ctx, GUIDE_E_ARG, "selection %u: constraint %u names an unknown column", i, k);
        if (!c.out.count) return fail(ctx, GUIDE_E_ARG, "selection %u: out.count is NULL", i);
        if (c.mode == GUIDE_SELECT_TOPK) {
            if (c.k == 0 || c.k > GUIDE_MAX_TOPK)
                return fail(ctx, GUIDE_E_ARG, "selection %u: k outside 1..%d", i, GUIDE_MAX_TOPK);
            if (!c.out.idx || !c.out.val) return fail(ctx, GUIDE_E_ARG, "selection %u: out.idx or out.val is NULL", i);
            topk = &c;
            // reduced inside the evaluation only when it has to be: a column it refers to is not stored
            topk_folded = can_fuse && c.k <= (uint32_t)kFusedTopK && !columns_present(c, *out);
        } else {
            if (c.out.capacity && !c.out.idx) return fail(ctx, GUIDE_E_ARG, "selection %u: out.idx is NULL", i);
            pareto = &c;
        }
        const bool reads_columns = count > 0 && !(c.mode == GUIDE_SELECT_TOPK && topk_folded);
        if (reads_columns && !columns_present(c, *out))
            return fail(ctx, GUIDE_E_ARG, "selection %u: a column it reads is not stored (NULL in guide_metrics)", i);
    }
    const size_t need = guide_eval_select_workspace_bytes(sel, n_sel, count);
    if (need && (!workspace || workspace_bytes < need))
        return fail(ctx, GUIDE_E_NOMEM, "workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    // workspace slices, in selection order
    void *ws_of[2] = {nullptr, nullptr};
    {
        char *p = (char *)workspace;
        for (uint32_t i = 0; i < n_sel; ++i) {
            ws_of[i] = p;
            p += guide_eval_select_workspace_bytes(sel + i, 1, count);
        }
    }
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return fail(ctx, GUIDE_E_DEVICE, "cannot select device %d", ctx->device);
    if (int rc_order = order_after_previous(ctx, stream)) return rc_order;
    uint32_t n_blocks = 0;
    bool sampled = false;                               // the evaluation kernel's extra blocks took the Pareto row sample
    bool eval_timed = false;
    // rows [0, count) of the columns are rows [first, first + count) of the grid: the chunks line up when first does
    const uint32_t chunk_of_eval = eval_grid_row_chunk(desc);
    const uint32_t row_chunk = (chunk_of_eval && first % chunk_of_eval == 0) ? chunk_of_eval : 0u;
    const bool fold = topk_folded;                      // then the Pareto row sample is taken there as well
    if (count > 0) {
        if (n_eff) {
            ctx->host_tab.eff_c[0] = eff->e_c[0];
            ctx->host_tab.eff_b[0] = eff->e_b[0];
        }
        rc = upload_grid_tables(ctx, desc, stream);
        if (rc) return rc;
        const double e_c = n_eff ? eff->e_c[0] : 1.0, e_b = n_eff ? eff->e_b[0] : 1.0;
        const bool additive = time_model == GUIDE_TIME_ADDITIVE;
        hipError_t e;
        const LaunchTiming timing = next_timing(ctx);
        eval_timed = timing.start != nullptr;
        if (fold) {
            FusedSelect fs;
            memset(&fs, 0, sizeof fs);
            fs.topk = 1;
            fs.topk_obj = topk->objective;
            fs.topk_filter = filter_of(*topk);
            fs.topk_ws = ws_of[topk - sel];
            if (pareto) {
                fs.pareto = 1;
                fs.pareto_x = pareto->objective;
                fs.pareto_y = pareto->objective_y;
                fs.pareto_filter = filter_of(*pareto);
                fs.scratch = ctx->select_scratch;
            }
            e = launch_eval_grid_fused(desc, ctx->dev_tab, ctx->dev_tile, (uint32_t)first, (uint32_t)count, e_c, e_b,
                                       additive, *out, fs, stream, &n_blocks, timing);
        } else if (pareto) {
            // the row sample of the Pareto selection is taken by extra blocks of the evaluation kernel
            FusedSelect fs;
            memset(&fs, 0, sizeof fs);
            fs.pareto = 1;
            fs.pareto_x = pareto->objective;
            fs.pareto_y = pareto->objective_y;
            fs.pareto_filter = filter_of(*pareto);
            fs.scratch = ctx->select_scratch;
            e = launch_eval_grid(desc, ctx->dev_tab, ctx->dev_tile, (uint32_t)first, (uint32_t)count, e_c, e_b, additive,
                                 *out, stream, timing, &fs, &sampled);
        } else {
            e = launch_eval_grid(desc, ctx->dev_tab, ctx->dev_tile, (uint32_t)first, (uint32_t)count, e_c, e_b, additive,
                                 *out, stream, timing);
        }
        if (e != hipSuccess) return hip_fail(ctx, e, "eval_select launch");
    }
    hipError_t e = hipSuccess;
    if (topk && pareto && count > 0 && !fold) {
        // both selections read stored columns: the small kernels ride along with the large ones
        // with a timed evaluation kernel, the two passes are timed as well (when the pairs suffice)
        LaunchTiming passes[2];
        const bool timed = eval_timed && pass_timing(ctx, passes);
        e = launch_select_both(spec_of(*topk, *out), topk->out, ws_of[topk - sel], spec_of(*pareto, *out), pareto->out,
                               ws_of[pareto - sel], count, ctx->select_scratch, stream, sampled, row_chunk,
                               timed ? passes : nullptr);
    } else {
        for (uint32_t i = 0; i < n_sel && e == hipSuccess; ++i) {
            const guide_column_select &c = sel[i];
            const guide_select_spec spec = spec_of(c, *out);
            if (c.mode == GUIDE_SELECT_TOPK) {
                if (!fold)
                    e = launch_select_topk(spec, count, c.out, ws_of[i], ctx->select_scratch, stream);
                else if (!pareto)
                    e = launch_topk_merge(ws_of[i], n_blocks, c.k, c.out, stream);
                // else: merged beside the Pareto front's finishing kernel, below
            } else if (fold) {
                e = launch_pareto_sampled(spec, count, c.out, ws_of[i], ctx->select_scratch, ws_of[topk - sel],
                                          n_blocks, topk->k, &topk->out, stream);
            } else if (sampled && count > 0) {
                e = launch_pareto_sampled(spec, count, c.out, ws_of[i], ctx->select_scratch, nullptr, 0,
                                          0, nullptr, stream, row_chunk);
            } else {
                e = launch_select_pareto(spec, count, c.out, ws_of[i], ctx->select_scratch, stream);
            }
        }
    }
    if (e != hipSuccess) return hip_fail(ctx, e, "eval_select selection launch");
    return GUIDE_OK;
}

int guide_profile_enable(guide_ctx *ctx, uint32_t capacity, uint32_t every) {
    if (!ctx) return GUIDE_E_ARG;
    if (capacity > (1u << 20)) return fail(ctx, GUIDE_E_RANGE, "more than 2^20 timed launches");
    if (capacity && every == 0) return fail(ctx, GUIDE_E_ARG, "every must be at least 1");
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return fail(ctx, GUIDE_E_DEVICE, "cannot select device %d", ctx->device);
    for (hipEvent_t e : ctx->prof_ev) (void)hipEventDestroy(e);
    ctx->prof_ev.clear();
    ctx->prof_used = 0;
    ctx->prof_seen = 0;
    ctx->prof_every = every ? every : 1;
    for (uint32_t i = 0; i < 2 * capacity; ++i) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return fail(ctx, GUIDE_E_DEVICE, "cannot create a timing event");
        ctx->prof_ev.push_back(e);
    }
    return GUIDE_OK;
}

int guide_profile_read(guide_ctx *ctx, float *ms, uint32_t *n) {
    if (!ctx) return GUIDE_E_ARG;
    if (!ms || !n) return fail(ctx, GUIDE_E_ARG, "ms or n is NULL");
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return fail(ctx, GUIDE_E_DEVICE, "cannot select device %d", ctx->device);
    for (uint32_t i = 0; i < ctx->prof_used; ++i) {
        GUIDE_HIP(ctx, hipEventSynchronize(ctx->prof_ev[2 * i + 1]));
        GUIDE_HIP(ctx, hipEventElapsedTime(&ms[i], ctx->prof_ev[2 * i], ctx->prof_ev[2 * i + 1]));
    }
    *n = ctx->prof_used;
    ctx->prof_used = 0;
    ctx->prof_seen = 0;
    return GUIDE_OK;
}

int guide_eval_extras(guide_ctx *ctx, const guide_grid *grid, uint64_t first, uint64_t count, uint32_t n_gpus,
                      uint32_t time_model, const guide_extras *out, void *stream_) {
    if (!ctx) return GUIDE_E_ARG;
    hipStream_t stream = (hipStream_t)stream_;
    if (!time_model_ok(time_model)) return fail(ctx, GUIDE_E_ARG, "unknown time model %u", time_model);
    if (!out) return fail(ctx, GUIDE_E_ARG, "guide_extras is NULL");
    if (n_gpus == 0) return fail(ctx, GUIDE_E_ARG, "n_gpus is zero");
    if (!(out->kv_keep >= 0.0 && out->kv_keep <= 1.0))
        return fail(ctx, GUIDE_E_ARG, "kv_keep must be in (0, 1] (or 0 for none), got %g", out->kv_keep);
    GridDesc desc;
    uint64_t size = 0;
    int rc = prepare_grid(ctx, grid, &desc, &size);
    if (rc) return rc;
    if (first > size || count > size - first)
        return fail(ctx, GUIDE_E_RANGE, "range [%llu, +%llu) outside the grid of %llu", (unsigned long long)first,
                    (unsigned long long)count, (unsigned long long)size);
    if (count == 0) return GUIDE_OK;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return fail(ctx, GUIDE_E_DEVICE, "cannot select device %d", ctx->device);
    if (int rc_order = order_after_previous(ctx, stream)) return rc_order;
    rc = upload_tables(ctx, stream);
    if (rc) return rc;
    const hipError_t e = launch_eval_extras(desc, ctx->dev_tab, (uint32_t)first, (uint32_t)count, n_gpus,
                                            time_model == GUIDE_TIME_ADDITIVE, *out, stream);
    if (e != hipSuccess) return hip_fail(ctx, e, "eval_extras launch");
    return GUIDE_OK;
}

size_t guide_select_workspace_bytes(const guide_select_spec *spec, uint64_t n) {
    if (!spec) return 0;
    return select_workspace_bytes(*spec, n);
}

// Argument checks shared by guide_select and guide_select_static.
static int check_select_args(guide_ctx *ctx, const guide_select_spec *spec, uint64_t n, const guide_select_out *out);

int guide_select_static(guide_ctx *ctx, const guide_select_spec *spec, uint64_t n, const guide_select_out *out,
                        void *stream_) {
    if (!ctx) return GUIDE_E_ARG;
    hipStream_t stream = (hipStream_t)stream_;
    const int rc = check_select_args(ctx, spec, n, out);
    if (rc) return rc;
    const size_t need = select_workspace_bytes(*spec, n);
    if (need > kStaticWsBytes)
        return fail(ctx, GUIDE_E_RANGE, "selection needs %zu bytes of workspace, the static scratch holds %zu "
                    "(Pareto: at most %llu rows)", need, kStaticWsBytes, (unsigned long long)GUIDE_STATIC_SELECT_MAX_ROWS);
    if (ctx->device >= kMaxDevices || !g_static_scratch[ctx->device])
        return fail(ctx, GUIDE_E_DEVICE, "no static scratch on device %d", ctx->device);
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return fail(ctx, GUIDE_E_DEVICE, "cannot select device %d", ctx->device);
    if (int rc_order = order_after_previous(ctx, stream)) return rc_order;
    unsigned char *base = (unsigned char *)g_static_scratch[ctx->device];
    void *tables = base, *workspace = base + kSelectScratchMax;
    const hipError_t e = spec->mode == GUIDE_SELECT_TOPK ? launch_select_topk(*spec, n, *out, workspace, tables, stream)
                                                         : launch_select_pareto(*spec, n, *out, workspace, tables, stream);
    if (e != hipSuccess) return hip_fail(ctx, e, "select launch");
    return GUIDE_OK;
}

int guide_select(guide_ctx *ctx, const guide_select_spec *spec, uint64_t n, const guide_select_out *out,
                 void *workspace, size_t workspace_bytes, void *stream_) {
    if (!ctx) return GUIDE_E_ARG;
    hipStream_t stream = (hipStream_t)stream_;
    const int rc_args = check_select_args(ctx, spec, n, out);
    if (rc_args) return rc_args;
    const size_t need = select_workspace_bytes(*spec, n);
    if (need && (!workspace || workspace_bytes < need))
        return fail(ctx, GUIDE_E_NOMEM, "workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return fail(ctx, GUIDE_E_DEVICE, "cannot select device %d", ctx->device);
    if (int rc_order = order_after_previous(ctx, stream)) return rc_order;
    const hipError_t e = spec->mode == GUIDE_SELECT_TOPK
                             ? launch_select_topk(*spec, n, *out, workspace, ctx->select_scratch, stream)
                             : launch_select_pareto(*spec, n, *out, workspace, ctx->select_scratch, stream);
    if (e != hipSuccess) return hip_fail(ctx, e, "select launch");
    return GUIDE_OK;
}

static int check_select_args(guide_ctx *ctx, const guide_select_spec *spec, uint64_t n, const guide_select_out *out) {
    if (!spec || !out) return fail(ctx, GUIDE_E_ARG, "spec or out is NULL");
    if (spec->mode != GUIDE_SELECT_TOPK && spec->mode != GUIDE_SELECT_PARETO)
        return fail(ctx, GUIDE_E_ARG, "unknown select mode %u", spec->mode);
    if (n > GUIDE_SELECT_MAX_ROWS)               // row indices are 32-bit and blocks read in units of 2048 rows
        return fail(ctx, GUIDE_E_RANGE, "more than 2^32 - 4096 rows");
    if (spec->n_constraints > GUIDE_MAX_CONSTRAINTS)
        return fail(ctx, GUIDE_E_ARG, "more than %d constraints", GUIDE_MAX_CONSTRAINTS);
    for (uint32_t c = 0; c < spec->n_constraints; ++c)
        if (!spec->constraints[c].column && n) return fail(ctx, GUIDE_E_ARG, "constraint %u: NULL column", c);
    if (!out->count) return fail(ctx, GUIDE_E_ARG, "out.count is NULL");
    if (n && !spec->objective) return fail(ctx, GUIDE_E_ARG, "objective is NULL");
    if (spec->mode == GUIDE_SELECT_TOPK) {
        if (spec->k == 0 || spec->k > GUIDE_MAX_TOPK) return fail(ctx, GUIDE_E_ARG, "k outside 1..%d", GUIDE_MAX_TOPK);
        if (spec->n_groups == 0 || spec->n_groups > GUIDE_MAX_GROUPS)
            return fail(ctx, GUIDE_E_ARG, "n_groups outside 1..%d", GUIDE_MAX_GROUPS);
        if (!out->idx || !out->val) return fail(ctx, GUIDE_E_ARG, "out.idx or out.val is NULL");
    } else {
        if (n && !spec->objective_y) return fail(ctx, GUIDE_E_ARG, "objective_y is NULL");
        if (out->capacity && !out->idx) return fail(ctx, GUIDE_E_ARG, "out.idx is NULL");
    }
    return GUIDE_OK;
}

int guide_eval_sampled(guide_ctx *ctx, const guide_space *space, uint64_t seed, uint64_t first, uint64_t count,
                       const double *bucket_edges, uint32_t n_edges, double ttft_cap, uint32_t time_model,
                       const guide_sampled_out *out, void *stream_) {
    if (!ctx) return GUIDE_E_ARG;
    hipStream_t stream = (hipStream_t)stream_;
    if (!time_model_ok(time_model)) return fail(ctx, GUIDE_E_ARG, "unknown time model %u", time_model);
    if (!space || !out) return fail(ctx, GUIDE_E_ARG, "space or out is NULL");
    if (!space->heads || !space->peak || !space->bw || !space->cap || !space->batch || !space->s_in || !space->s_out ||
        !space->tp || !space->wbits || !space->kv_block || !space->mbt || !space->kv_choices)
        return fail(ctx, GUIDE_E_ARG, "space has a NULL table");
    if (n_edges > GUIDE_MAX_BUCKET_EDGES || (n_edges && !bucket_edges))
        return fail(ctx, GUIDE_E_ARG, "bucket edges: need 0..%d", GUIDE_MAX_BUCKET_EDGES);
    if (!out->feasible_count || !out->win_val || !out->win_idx || !out->hist)
        return fail(ctx, GUIDE_E_ARG, "a reduced output pointer is NULL");
    if (count > (1ull << 40) || first > UINT64_MAX - count) return fail(ctx, GUIDE_E_RANGE, "count too large");
    if (space->layers_n == 0 || space->layers_n > 65536 || !(space->link_div > 0.0) || space->vocab == 0)
        return fail(ctx, GUIDE_E_ARG, "space: bad scalar field");
    SpaceTables *t = new (std::nothrow) SpaceTables;
    if (!t) return fail(ctx, GUIDE_E_NOMEM, "host allocation failed");
    memset(t, 0, sizeof *t);
    memcpy(t->heads, space->heads, sizeof t->heads);
    memcpy(t->batch, space->batch, sizeof t->batch);
    memcpy(t->s_in, space->s_in, sizeof t->s_in);
    memcpy(t->s_out, space->s_out, sizeof t->s_out);
    memcpy(t->peak, space->peak, sizeof t->peak);
    memcpy(t->bw, space->bw, sizeof t->bw);
    memcpy(t->cap, space->cap, sizeof(double) * 6);
    memcpy(t->tp, space->tp, sizeof(uint32_t) * 4);
    memcpy(t->wbits, space->wbits, sizeof(uint32_t) * 3);
    memcpy(t->kv_block, space->kv_block, sizeof(uint32_t) * 2);
    memcpy(t->mbt, space->mbt, sizeof(uint32_t) * 3);
    memcpy(t->kv_choices, space->kv_choices, sizeof(uint32_t) * 4);
    for (uint32_t i = 0; i < n_edges; ++i) t->edges[i] = bucket_edges[i];
    t->n_edges = n_edges;
    t->layers_lo = space->layers_lo; t->layers_n = space->layers_n;
    t->ffn_lo_x2 = space->ffn_lo_x2; t->ffn_span_x2 = space->ffn_span_x2;
    t->vocab = space->vocab; t->link_div = space->link_div;
    int rc = GUIDE_OK;
    for (uint32_t i = 0; i < GUIDE_LATTICE && rc == GUIDE_OK; ++i) {
        if (t->heads[i] == 0 || t->heads[i] > 1024 || !t->batch[i] || !t->s_in[i] || !t->s_out[i] ||
            t->s_in[i] > 0x7FFFFFFFu || t->s_out[i] > 0x7FFFFFFFu || !(t->peak[i] > 0.0) || !(t->bw[i] > 0.0))
            rc = fail(ctx, GUIDE_E_ARG, "space: bad lattice entry %u", i);
    }
    for (uint32_t i = 0; i < 4 && rc == GUIDE_OK; ++i)
        if (!t->tp[i] || (i < 3 && (!t->wbits[i] || !t->mbt[i])) || (i < 2 && !t->kv_block[i]))
            rc = fail(ctx, GUIDE_E_ARG, "space: zero knob value");
    if (rc) { delete t; return rc; }
    DeviceGuard guard(ctx->device);
    if (!guard.ok) { delete t; return fail(ctx, GUIDE_E_DEVICE, "cannot select device %d", ctx->device); }
    rc = order_after_previous(ctx, stream);
    if (rc) { delete t; return rc; }
    rc = stage_upload(ctx, ctx->dev_space, t, sizeof(SpaceTables), stream);
    delete t;
    if (rc) return rc;
    hipError_t e = launch_eval_sampled(ctx->dev_space, seed, first, count, ttft_cap, time_model == GUIDE_TIME_ADDITIVE, *out,
                            ctx->sampled_scratch, stream, n_edges);
    if (e != hipSuccess) return hip_fail(ctx, e, "eval_sampled launch");
    return GUIDE_OK;
}

size_t guide_simulate_workspace_bytes(uint32_t n_cfg, uint32_t n_requests) {
    return simulate_workspace_bytes(n_cfg, n_requests);
}

int guide_simulate(guide_ctx *ctx, const guide_grid *grid, const uint32_t *cfg_idx, const double *rate, uint32_t n_cfg,
                   const guide_trace *trace, uint32_t time_model, uint32_t scheduler, const guide_sim_out *out,
                   void *workspace, size_t workspace_bytes, void *stream_) {
    if (!ctx) return GUIDE_E_ARG;
    hipStream_t stream = (hipStream_t)stream_;
    if (!time_model_ok(time_model)) return fail(ctx, GUIDE_E_ARG, "unknown time model %u", time_model);
    const bool closed_runs = (scheduler & GUIDE_SIM_CLOSED_FORM_RUNS) != 0;
    scheduler &= ~(uint32_t)GUIDE_SIM_CLOSED_FORM_RUNS;
    if (scheduler != GUIDE_SCHED_SPLIT_FUSE && scheduler != GUIDE_SCHED_PREFILL_FIRST)
        return fail(ctx, GUIDE_E_ARG, "unknown scheduler %u", scheduler);
    if (!trace || !out) return fail(ctx, GUIDE_E_ARG, "trace or out is NULL");
    if (trace->n == 0 || trace->n > GUIDE_MAX_REQUESTS)
        return fail(ctx, GUIDE_E_RANGE, "trace: need 1..%d requests", GUIDE_MAX_REQUESTS);
    if (!trace->arrival_unit || !trace->n_in || !trace->n_out) return fail(ctx, GUIDE_E_ARG, "trace has a NULL array");
    if (!out->ttft_p50 || !out->ttft_p99 || !out->mean_tpot || !out->tokens_s || !out->status || !out->n_steps ||
        !out->n_request_steps)
        return fail(ctx, GUIDE_E_ARG, "an output pointer is NULL");
    GridDesc desc;
    uint64_t size = 0;
    int rc = prepare_grid(ctx, grid, &desc, &size);
    if (rc) return rc;
    if (n_cfg == 0) return GUIDE_OK;
    if (!cfg_idx || !rate) return fail(ctx, GUIDE_E_ARG, "cfg_idx or rate is NULL");
    TraceDev *t = new (std::nothrow) TraceDev;
    if (!t) return fail(ctx, GUIDE_E_NOMEM, "host allocation failed");
    memset(t, 0, sizeof *t);
    double prev = -INFINITY, sum_in = 0.0, sum_out = 0.0;
    for (uint32_t i = 0; i < trace->n && rc == GUIDE_OK; ++i) {
        const double a = trace->arrival_unit[i];
        if (!(a >= 0.0) || std::isinf(a) || a < prev) rc = fail(ctx, GUIDE_E_ARG, "trace: arrival %u not non-decreasing / finite", i);
        if (trace->n_in[i] == 0 || trace->n_out[i] == 0 || trace->n_in[i] > (1u << 24) || trace->n_out[i] > (1u << 24))
            rc = fail(ctx, GUIDE_E_ARG, "trace: request %u has a length outside 1..2^24", i);
        prev = a;
        t->arrival[i] = a; t->n_in[i] = trace->n_in[i]; t->n_out[i] = trace->n_out[i];
        sum_in += (double)trace->n_in[i];
        sum_out += (double)trace->n_out[i];
    }
    if (rc) { delete t; return rc; }
    const size_t need = simulate_workspace_bytes(n_cfg, trace->n);
    if (!workspace || workspace_bytes < need) {
        delete t;
        return fail(ctx, GUIDE_E_NOMEM, "workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    }
    DeviceGuard guard(ctx->device);
    if (!guard.ok) { delete t; return fail(ctx, GUIDE_E_DEVICE, "cannot select device %d", ctx->device); }
    rc = order_after_previous(ctx, stream);
    if (rc) { delete t; return rc; }
    rc = stage_upload(ctx, ctx->dev_trace, t, sizeof(TraceDev), stream);
    delete t;
    if (rc) return rc;
    rc = upload_tables(ctx, stream);
    if (rc) return rc;
    hipError_t e = launch_simulate(desc, ctx->dev_tab, ctx->dev_trace, trace->n, cfg_idx, rate, n_cfg,
                        time_model == GUIDE_TIME_ADDITIVE, scheduler == GUIDE_SCHED_PREFILL_FIRST, closed_runs, *out, workspace,
                        stream, sum_in, sum_out);
    if (e != hipSuccess) return hip_fail(ctx, e, "simulate launch");
    return GUIDE_OK;
}

}  // extern "C"
