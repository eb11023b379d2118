// Launchers implemented in the kernel translation units, called by the C ABI.
#pragma once

#include "common.hpp"

namespace guide {

hipError_t launch_eval_grid(const GridDesc &g, const DevTables *tab, uint32_t first, uint32_t count, double e_c,
                            double e_b, bool additive, const guide_metrics &out, hipStream_t stream);
hipError_t launch_eval_sweep(const GridDesc &g, const DevTables *tab, uint32_t first, uint32_t count, uint32_t n_eff,
                             bool additive, const guide_stats &out, hipStream_t stream);

size_t select_workspace_bytes(const guide_select_spec &spec, uint64_t n);
hipError_t launch_eval_extras(const GridDesc &g, const DevTables *tab, uint32_t first, uint32_t count, uint32_t n_gpus,
                              bool additive, const guide_extras &out, hipStream_t stream);

size_t select_scratch_bytes();
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
                           bool prefill_first, const guide_sim_out &out, void *ws, hipStream_t stream);

}  // namespace guide
