// Launchers implemented in the kernel translation units, called by the C ABI.
#pragma once

#include "common.hpp"

namespace guide {

// Tables derived from (grid description, device tables) that the tile kernels copy into LDS; they
// are recomputed by launch_tile_tables whenever either changes.
size_t tile_tables_bytes();
hipError_t launch_tile_tables(const GridDesc &g, const DevTables *tab, void *tile_tables, hipStream_t stream);
// Events that receive the start and the end of the evaluation kernel itself (attached to its dispatch),
// or nullptr.
struct LaunchTiming {
    hipEvent_t start = nullptr, stop = nullptr;
};
hipError_t launch_eval_sweep(const GridDesc &g, const DevTables *tab, uint32_t first, uint32_t count, uint32_t n_eff,
                             bool additive, const guide_stats &out, hipStream_t stream);

// Selections folded into the grid evaluation (guide_eval_select): while a row's values are still
// in registers the evaluation feeds a per-lane top-K list and / or the row sample that fixes the
// bin range of the Pareto kernels, so neither needs a pass of its own over the columns.
constexpr int kFusedTopK = 4;
struct FusedFilter {
    uint32_t use_feasible, n_con;
    uint32_t col[GUIDE_MAX_CONSTRAINTS];        // GUIDE_COL_*
    double cap[GUIDE_MAX_CONSTRAINTS];
};
struct FusedSelect {
    // rider_blocks != 0: that many extra blocks at the end of the grid take the row sample of a Pareto selection
    // over the evaluated rows (pareto_x, pareto_y, pareto_filter, scratch below) by evaluating the sampled rows
    // themselves, beside the blocks that evaluate and store the grid.
    uint32_t rider_blocks;
    uint32_t topk, topk_obj;                    // topk != 0: least kFusedTopK rows by column topk_obj
    FusedFilter topk_filter;
    void *topk_ws;                              // block partials, layout of the top-k pass
    uint32_t pareto, pareto_x, pareto_y;        // pareto != 0: a Pareto selection over (x, y) follows: take its row sample
    FusedFilter pareto_filter;
    void *scratch;                              // scratch of the Pareto kernels
};
// sample != nullptr (grids with a tile kernel only): extra blocks take the row sample of the Pareto selection that
// sample->pareto_* describe; *sampled tells whether they did.
hipError_t launch_eval_grid(const GridDesc &g, const DevTables *tab, const void *tile_tables, uint32_t first,
                            uint32_t count, double e_c, double e_b, bool additive, const guide_metrics &out,
                            hipStream_t stream, LaunchTiming timing = LaunchTiming(), const FusedSelect *sample = nullptr,
                            bool *sampled = nullptr);
// True when the grid's two fastest axes have a compiled tile kernel (the only one that folds selections in).
bool eval_grid_can_fuse(const GridDesc &g);
// The evaluation with a top-k folded in (and the row sample of fs.pareto taken by extra blocks); *n_blocks
// receives the number of blocks that wrote top-k partials.
hipError_t launch_eval_grid_fused(const GridDesc &g, const DevTables *tab, const void *tile_tables, uint32_t first,
                                  uint32_t count, double e_c, double e_b, bool additive, const guide_metrics &out,
                                  const FusedSelect &fs, hipStream_t stream, uint32_t *n_blocks,
                                  LaunchTiming timing = LaunchTiming());
// Second halves of the folded selections.
hipError_t launch_topk_merge(void *ws, uint32_t n_blocks, uint32_t k, const guide_select_out &out, hipStream_t stream);
hipError_t launch_pareto_sampled(const guide_select_spec &spec, uint64_t n, const guide_select_out &out, void *ws,
                                 void *scratch, void *merge_ws, uint32_t merge_blocks,
                                 uint32_t merge_k, const guide_select_out *merge_out, hipStream_t stream,
                                 uint32_t row_chunk = 0);
size_t topk_partials_bytes();
// sampled: the caller's evaluation kernel has already taken the row sample, so none is launched.
hipError_t launch_select_both(const guide_select_spec &topk, const guide_select_out &topk_out, void *topk_ws,
                              const guide_select_spec &pareto, const guide_select_out &pareto_out, void *pareto_ws,
                              uint64_t n, void *scratch, hipStream_t stream, bool sampled = false,
                              uint32_t row_chunk = 0, const LaunchTiming *pass_timing = nullptr);
// pass_timing: two event pairs for the filter and finishing kernels (or nullptr).
// row_chunk: rows are dealt to the blocks of the selection passes in chunks of that many rows, chunk c to block
// c % blocks (0 = the passes' own batch size).  eval_grid_row_chunk() gives the chunk in which the evaluation
// kernel deals its rows to blocks the same way, so that a row is read through the L2 that wrote it.
uint32_t eval_grid_row_chunk(const GridDesc &g);

size_t select_workspace_bytes(const guide_select_spec &spec, uint64_t n);
hipError_t launch_eval_extras(const GridDesc &g, const DevTables *tab, uint32_t first, uint32_t count, uint32_t n_gpus,
                              bool additive, const guide_extras &out, hipStream_t stream);

size_t select_scratch_bytes();
constexpr size_t kSelectScratchMax = 128 * 1024;   // upper bound of select_scratch_bytes(), for static storage
hipError_t launch_select_topk(const guide_select_spec &spec, uint64_t n, const guide_select_out &out, void *ws,
                              void *scratch, hipStream_t stream);
hipError_t launch_select_pareto(const guide_select_spec &spec, uint64_t n, const guide_select_out &out, void *ws,
                                void *scratch, hipStream_t stream);

// Device tables of the sampled space (built from the HOST guide_space).
struct SpaceTables {
    uint32_t heads[GUIDE_LATTICE], batch[GUIDE_LATTICE], s_in[GUIDE_LATTICE], s_out[GUIDE_LATTICE];
    double peak[GUIDE_LATTICE], bw[GUIDE_LATTICE];
    double cap[8];
    double edges[GUIDE_MAX_BUCKET_EDGES + 1];
    uint32_t tp[4], wbits[4], kv_block[2], mbt[4], kv_choices[4];
    uint32_t layers_lo, layers_n, ffn_lo_x2, ffn_span_x2, vocab, n_edges;
    double link_div;     // link_bw = bw / link_div
};
constexpr uint32_t kSampledMaxBlocks = 2048;
size_t sampled_scratch_bytes();
hipError_t launch_eval_sampled(const SpaceTables *tab, uint64_t seed, uint64_t first, uint64_t count, double ttft_cap,
                               bool additive, const guide_sampled_out &out, void *scratch, hipStream_t stream,
                               uint32_t n_edges);

size_t simulate_workspace_bytes(uint32_t n_cfg, uint32_t n_req);
struct TraceDev {
    double arrival[GUIDE_MAX_REQUESTS];
    uint32_t n_in[GUIDE_MAX_REQUESTS];
    uint32_t n_out[GUIDE_MAX_REQUESTS];
};
hipError_t launch_simulate(const GridDesc &g, const DevTables *tab, const TraceDev *trace, uint32_t n_req,
                           const uint32_t *cfg_idx, const double *rate, uint32_t n_cfg, bool additive,
                           bool prefill_first, bool closed_runs, const guide_sim_out &out, void *ws, hipStream_t stream,
                           double sum_in, double sum_out);   // sums of the trace's prompt / generated tokens

}  // namespace guide
