#include "kernels.hpp"
namespace guide {
size_t simulate_workspace_bytes(uint32_t, uint32_t) { return 256; }
hipError_t launch_simulate(const GridDesc &, const DevTables *, const TraceDev *, uint32_t, const uint32_t *,
                           const double *, uint32_t, bool, const guide_sim_out &, void *, hipStream_t) { return hipErrorNotSupported; }
}
