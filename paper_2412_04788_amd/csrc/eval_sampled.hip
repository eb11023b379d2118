#include "kernels.hpp"
namespace guide {
size_t sampled_scratch_bytes() { return 256; }
hipError_t launch_eval_sampled(const SpaceTables *, uint64_t, uint64_t, uint64_t, double, bool, const guide_sampled_out &,
                               void *, hipStream_t) { return hipErrorNotSupported; }
}
