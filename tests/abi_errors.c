/*
 * Drives the error paths of the C ABI (include/guide.h) from plain C: NULL pointers, zero counts, unknown enums,
 * ranges and sizes beyond the stated limits.  Every call must return its status code without crashing, enqueue
 * nothing, and leave a message in guide_last_error().  Without a GPU (argument "nogpu") only the paths that need no
 * context run.  Device pointers are never dereferenced by a rejected call, so dummy values stand in for them.
 * Prints one line per check; exit status 0 when all hold.
 */
#include <stdio.h>
#include <string.h>

#include "guide.h"

static int failures = 0;
#define EXPECT(call, code)                                                                    \
    do {                                                                                      \
        int rc_ = (call);                                                                     \
        if (rc_ != (code)) { printf("FAIL %s -> %d, expected %d\n", #call, rc_, (code)); ++failures; } \
        else printf("ok   %s -> %d\n", #call, rc_);                                           \
    } while (0)

int main(int argc, char **argv) {
    const int nogpu = argc > 1 && strcmp(argv[1], "nogpu") == 0;
    guide_ctx *ctx = NULL;
    uint64_t vals[2] = {16, 32}, one[1] = {1}, zero[1] = {0}, big[1] = {0x7FFFFFFFull}, huge[1] = {0xFFFFFFFFull};
    guide_axis a1 = {1, GUIDE_AXIS_TABLE, 0, one}, idx0 = {1, GUIDE_AXIS_TABLE, 0, zero};
    guide_grid grid = {idx0, idx0, a1, a1, a1, a1, {1, GUIDE_AXIS_TABLE, 0, vals}, {2, GUIDE_AXIS_TABLE, 0, vals}, a1};
    guide_model model = {32, 4096, 32, 32, 11008, 32000, 1, 1};
    guide_hw hw = {1e15, 5e12, 2e11, 4e11, 0.0};
    double dummy_f64[8];
    uint64_t dummy_u64[8];
    guide_metrics out;
    memset(&out, 0, sizeof out);
    out.t_batch = dummy_f64;

    /* no context */
    EXPECT(guide_create(NULL, 0), GUIDE_E_ARG);
    EXPECT(guide_create(&ctx, -1), GUIDE_E_DEVICE);
    EXPECT(guide_create(&ctx, 4096), GUIDE_E_DEVICE);
    EXPECT(guide_set_models(NULL, &model, 1), GUIDE_E_ARG);
    EXPECT(guide_set_hardware(NULL, &hw, 1), GUIDE_E_ARG);
    EXPECT(guide_eval_grid(NULL, &grid, 0, 1, NULL, GUIDE_TIME_ROOFLINE, &out, NULL, NULL), GUIDE_E_ARG);
    EXPECT(guide_eval_extras(NULL, &grid, 0, 1, 8, 0, NULL, NULL), GUIDE_E_ARG);
    EXPECT(guide_select(NULL, NULL, 0, NULL, NULL, 0, NULL), GUIDE_E_ARG);
    EXPECT(guide_select_static(NULL, NULL, 0, NULL, NULL), GUIDE_E_ARG);
    EXPECT(guide_simulate(NULL, &grid, NULL, NULL, 0, NULL, 0, 0, NULL, NULL, 0, NULL), GUIDE_E_ARG);
    EXPECT(guide_eval_sampled(NULL, NULL, 0, 0, 0, NULL, 0, 0.2, 0, NULL, NULL), GUIDE_E_ARG);
    EXPECT(guide_eval_select(NULL, &grid, 0, 1, NULL, 0, &out, NULL, 0, NULL, 0, NULL), GUIDE_E_ARG);
    EXPECT(guide_profile_enable(NULL, 1, 1), GUIDE_E_ARG);
    EXPECT((int)guide_select_workspace_bytes(NULL, 10), 0);
    EXPECT((int)guide_eval_select_workspace_bytes(NULL, 1, 10), 0);
    EXPECT(guide_last_error(NULL) != NULL ? 0 : 1, 0);
    guide_destroy(NULL);
    if (nogpu) {
        EXPECT(guide_create(&ctx, 0), GUIDE_E_DEVICE);
        EXPECT(ctx == NULL ? 0 : 1, 0);
        printf("%d failure(s)\n", failures);
        return failures != 0;
    }

    EXPECT(guide_create(&ctx, 0), GUIDE_OK);
    /* tables */
    EXPECT(guide_eval_grid(ctx, &grid, 0, 1, NULL, 0, &out, NULL, NULL), GUIDE_E_ARG);      /* nothing registered yet */
    EXPECT(guide_set_models(ctx, NULL, 1), GUIDE_E_ARG);
    EXPECT(guide_set_models(ctx, &model, 0), GUIDE_E_ARG);
    EXPECT(guide_set_models(ctx, &model, GUIDE_MAX_MODELS + 1), GUIDE_E_ARG);
    { guide_model bad = model; bad.n_h = 33; EXPECT(guide_set_models(ctx, &bad, 1), GUIDE_E_ARG); }
    { guide_model bad = model; bad.k = 2; EXPECT(guide_set_models(ctx, &bad, 1), GUIDE_E_ARG); }
    { guide_hw bad = hw; bad.hbm_bw = 0.0; EXPECT(guide_set_hardware(ctx, &bad, 1), GUIDE_E_ARG); }
    EXPECT(guide_set_models(ctx, &model, 1), GUIDE_OK);
    EXPECT(guide_set_hardware(ctx, &hw, 1), GUIDE_OK);
    /* grid evaluation */
    EXPECT(guide_eval_grid(ctx, NULL, 0, 1, NULL, 0, &out, NULL, NULL), GUIDE_E_ARG);
    EXPECT(guide_eval_grid(ctx, &grid, 0, 1, NULL, 7, &out, NULL, NULL), GUIDE_E_ARG);     /* unknown time model */
    EXPECT(guide_eval_grid(ctx, &grid, 0, 1, NULL, 0, NULL, NULL, NULL), GUIDE_E_ARG);
    EXPECT(guide_eval_grid(ctx, &grid, 3, 2, NULL, 0, &out, NULL, NULL), GUIDE_E_RANGE);   /* grid has 2 rows */
    EXPECT(guide_eval_grid(ctx, &grid, 0, 0, NULL, 0, &out, NULL, NULL), GUIDE_OK);        /* count 0: no-op */
    { guide_grid g2 = grid; g2.batch.count = 0; EXPECT(guide_eval_grid(ctx, &g2, 0, 1, NULL, 0, &out, NULL, NULL), GUIDE_E_ARG); }
    { guide_grid g2 = grid; g2.tp.kind = 9; EXPECT(guide_eval_grid(ctx, &g2, 0, 1, NULL, 0, &out, NULL, NULL), GUIDE_E_ARG); }
    { guide_grid g2 = grid; g2.mbt.values = NULL; EXPECT(guide_eval_grid(ctx, &g2, 0, 1, NULL, 0, &out, NULL, NULL), GUIDE_E_ARG); }
    { guide_grid g2 = grid; g2.s_in.values = zero; EXPECT(guide_eval_grid(ctx, &g2, 0, 1, NULL, 0, &out, NULL, NULL), GUIDE_E_ARG); }
    { guide_grid g2 = grid; g2.model.values = one; EXPECT(guide_eval_grid(ctx, &g2, 0, 1, NULL, 0, &out, NULL, NULL), GUIDE_E_RANGE); }
    { guide_grid g2 = grid; g2.s_in.values = huge; EXPECT(guide_eval_grid(ctx, &g2, 0, 1, NULL, 0, &out, NULL, NULL), GUIDE_E_RANGE); }
    {   /* s_in + s_out + kv_block reaches 2^32 */
        guide_grid g2 = grid; g2.s_in.values = big; g2.s_out.values = big; g2.kv_block.count = 1; g2.kv_block.values = big;
        EXPECT(guide_eval_grid(ctx, &g2, 0, 1, NULL, 0, &out, NULL, NULL), GUIDE_E_RANGE);
    }
    { double e[2] = {1.0, -1.0}; guide_eff eff = {2, e, e}; guide_stats st; memset(&st, 0, sizeof st);
      EXPECT(guide_eval_grid(ctx, &grid, 0, 1, &eff, 0, &out, &st, NULL), GUIDE_E_ARG); }
    { double e[1] = {1.0}; guide_eff eff = {GUIDE_MAX_EFF + 1, e, e};
      EXPECT(guide_eval_grid(ctx, &grid, 0, 1, &eff, 0, &out, NULL, NULL), GUIDE_E_RANGE); }
    { double e[2] = {1.0, 1.0}; guide_eff eff = {2, e, e};
      EXPECT(guide_eval_grid(ctx, &grid, 0, 1, &eff, 0, &out, NULL, NULL), GUIDE_E_ARG); }    /* sweep without guide_stats */
    EXPECT(guide_eval_extras(ctx, &grid, 0, 1, 0, 0, NULL, NULL), GUIDE_E_ARG);
    { guide_extras ex; memset(&ex, 0, sizeof ex);
      ex.kv_keep = 1.5; EXPECT(guide_eval_extras(ctx, &grid, 0, 1, 8, 0, &ex, NULL), GUIDE_E_ARG);
      ex.kv_keep = -0.25; EXPECT(guide_eval_extras(ctx, &grid, 0, 1, 8, 0, &ex, NULL), GUIDE_E_ARG);
      ex.kv_keep = 0.0; EXPECT(guide_eval_extras(ctx, &grid, 0, 0, 8, 0, &ex, NULL), GUIDE_OK); }      /* no rows: no-op */
    /* selection */
    {
        guide_select_spec sp; guide_select_out so = {dummy_u64, dummy_f64, dummy_u64, 0};
        memset(&sp, 0, sizeof sp);
        sp.mode = 5; sp.objective = dummy_f64; sp.k = 1; sp.n_groups = 1;
        EXPECT(guide_select(ctx, &sp, 4, &so, dummy_u64, 1 << 20, NULL), GUIDE_E_ARG);
        sp.mode = GUIDE_SELECT_TOPK; sp.k = 0;
        EXPECT(guide_select(ctx, &sp, 4, &so, dummy_u64, 1 << 20, NULL), GUIDE_E_ARG);
        sp.k = GUIDE_MAX_TOPK + 1;
        EXPECT(guide_select(ctx, &sp, 4, &so, dummy_u64, 1 << 20, NULL), GUIDE_E_ARG);
        sp.k = 1; sp.n_groups = GUIDE_MAX_GROUPS + 1;
        EXPECT(guide_select(ctx, &sp, 4, &so, dummy_u64, 1 << 20, NULL), GUIDE_E_ARG);
        sp.n_groups = 1; sp.n_constraints = GUIDE_MAX_CONSTRAINTS + 1;
        EXPECT(guide_select(ctx, &sp, 4, &so, dummy_u64, 1 << 20, NULL), GUIDE_E_ARG);
        sp.n_constraints = 1;                                                       /* NULL constraint column */
        EXPECT(guide_select(ctx, &sp, 4, &so, dummy_u64, 1 << 20, NULL), GUIDE_E_ARG);
        sp.n_constraints = 0;
        EXPECT(guide_select(ctx, &sp, GUIDE_SELECT_MAX_ROWS + 1, &so, dummy_u64, 1 << 20, NULL), GUIDE_E_RANGE);
        EXPECT(guide_select(ctx, &sp, 4, &so, NULL, 0, NULL), GUIDE_E_NOMEM);
        EXPECT(guide_select(ctx, &sp, 4, &so, dummy_u64, 8, NULL), GUIDE_E_NOMEM);
        so.count = NULL;
        EXPECT(guide_select(ctx, &sp, 4, &so, dummy_u64, 1 << 20, NULL), GUIDE_E_ARG);
        so.count = dummy_u64; sp.mode = GUIDE_SELECT_PARETO;                         /* Pareto without objective_y */
        EXPECT(guide_select(ctx, &sp, 4, &so, dummy_u64, 1 << 20, NULL), GUIDE_E_ARG);
        sp.objective_y = dummy_f64;
        EXPECT(guide_select_static(ctx, &sp, GUIDE_STATIC_SELECT_MAX_ROWS + 1, &so, NULL), GUIDE_E_RANGE);
    }
    /* simulation */
    {
        double arr[2] = {0.0, 1.0}, arr_bad[2] = {1.0, 0.0};
        uint32_t nin[2] = {8, 8}, nout[2] = {4, 4}, nout0[2] = {4, 0};
        guide_trace tr = {2, arr, nin, nout};
        guide_sim_out so; memset(&so, 0, sizeof so);
        EXPECT(guide_simulate(ctx, &grid, NULL, NULL, 1, &tr, 0, 0, &so, dummy_u64, 1 << 20, NULL), GUIDE_E_ARG);  /* NULL outputs */
        so.ttft_p50 = so.ttft_p99 = so.mean_tpot = so.tokens_s = dummy_f64;
        so.status = (uint32_t *)dummy_u64; so.n_steps = so.n_request_steps = dummy_u64;
        EXPECT(guide_simulate(ctx, &grid, NULL, NULL, 1, &tr, 0, 9, &so, dummy_u64, 1 << 20, NULL), GUIDE_E_ARG);  /* scheduler */
        EXPECT(guide_simulate(ctx, &grid, NULL, NULL, 1, &tr, 0, 0, &so, dummy_u64, 1 << 20, NULL), GUIDE_E_ARG);  /* NULL cfg */
        EXPECT(guide_simulate(ctx, &grid, (uint32_t *)dummy_u64, dummy_f64, 1, &tr, 0, 0, &so, dummy_u64, 16, NULL), GUIDE_E_NOMEM);
        tr.arrival_unit = arr_bad;
        EXPECT(guide_simulate(ctx, &grid, (uint32_t *)dummy_u64, dummy_f64, 1, &tr, 0, 0, &so, dummy_u64, 1 << 20, NULL), GUIDE_E_ARG);
        tr.arrival_unit = arr; tr.n_out = nout0;
        EXPECT(guide_simulate(ctx, &grid, (uint32_t *)dummy_u64, dummy_f64, 1, &tr, 0, 0, &so, dummy_u64, 1 << 20, NULL), GUIDE_E_ARG);
        tr.n_out = nout; tr.n = GUIDE_MAX_REQUESTS + 1;
        EXPECT(guide_simulate(ctx, &grid, (uint32_t *)dummy_u64, dummy_f64, 1, &tr, 0, 0, &so, dummy_u64, 1 << 20, NULL), GUIDE_E_RANGE);
        tr.n = 2;
        EXPECT(guide_simulate(ctx, &grid, NULL, NULL, 0, &tr, 0, 0, &so, NULL, 0, NULL), GUIDE_OK);               /* no configurations */
    }
    /* evaluate and select */
    {
        guide_column_select cs; memset(&cs, 0, sizeof cs);
        cs.mode = GUIDE_SELECT_TOPK; cs.objective = GUIDE_NUM_COLS; cs.k = 1;
        cs.out.idx = dummy_u64; cs.out.val = dummy_f64; cs.out.count = dummy_u64;
        EXPECT(guide_eval_select(ctx, &grid, 0, 2, NULL, 0, &out, &cs, 1, dummy_u64, 1 << 20, NULL), GUIDE_E_ARG);   /* column id */
        cs.objective = GUIDE_COL_T_BATCH;
        EXPECT(guide_eval_select(ctx, &grid, 0, 2, NULL, 0, &out, &cs, 3, dummy_u64, 1 << 20, NULL), GUIDE_E_ARG);   /* n_sel */
        EXPECT(guide_eval_select(ctx, &grid, 0, 2, NULL, 0, &out, &cs, 1, NULL, 0, NULL), GUIDE_E_NOMEM);
        cs.mode = GUIDE_SELECT_PARETO; cs.objective_y = GUIDE_COL_COST;                                        /* cost column not stored */
        EXPECT(guide_eval_select(ctx, &grid, 0, 2, NULL, 0, &out, &cs, 1, dummy_u64, 1 << 26, NULL), GUIDE_E_ARG);
    }
    EXPECT(strlen(guide_last_error(ctx)) > 0 ? 0 : 1, 0);
    guide_destroy(ctx);
    printf("%d failure(s)\n", failures);
    return failures != 0;
}
