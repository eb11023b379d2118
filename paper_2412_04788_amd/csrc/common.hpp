// Shared host/device declarations of libguide (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "guide.h"

namespace guide {

constexpr int kWave = 64;          // CDNA wavefront width
constexpr int kBlock = 256;        // threads per workgroup (4 waves, one per SIMD)
constexpr int kNumAxes = 9;
constexpr int kNumCU = 256;        // MI355X compute units (a partitioned GPU reports fewer: see device_cus)

// Compute units of the current device, for sizing persistent launches; kNumCU when the query fails.
inline uint32_t device_cus() {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
        return (uint32_t)kNumCU;
    return (uint32_t)n;
}

enum AxisId { AX_MODEL = 0, AX_HW, AX_BATCH, AX_SIN, AX_SOUT, AX_TP, AX_WBITS, AX_BLK, AX_MBT };

// Exact unsigned division of a 32-bit value by an invariant divisor
// (Granlund & Montgomery, "Division by invariant integers using multiplication",
// PLDI'94, unsigned case with N = 32): q = (t + ((n - t) >> s1)) >> s2 with
// t = mulhi(m, n).
struct Div32 {
    uint32_t m, s1, s2, d;
};

__host__ __device__ inline Div32 make_div32(uint32_t d) {
    Div32 r;
    r.d = d;
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;   // ceil(log2 d)
    r.m = (uint32_t)(((1ull << 32) * ((1ull << l) - d)) / d + 1);
    r.s1 = l < 1 ? l : 1;
    r.s2 = l > 0 ? l - 1 : 0;
    return r;
}

__host__ __device__ inline uint32_t div32(uint32_t n, const Div32 &dv) {
#if defined(__HIP_DEVICE_COMPILE__)
    uint32_t t = __umulhi(dv.m, n);
#else
    uint32_t t = (uint32_t)(((uint64_t)dv.m * n) >> 32);
#endif
    return (t + ((n - t) >> dv.s1)) >> dv.s2;
}

// Launch description of a grid: radices with their dividers (fastest axis last).
struct GridDesc {
    Div32 div[kNumAxes];
    uint32_t n_models, n_hw;
};

// Device-resident tables of one context (uploaded per call, stream ordered).
struct DevTables {
    uint32_t axis_vals[kNumAxes][GUIDE_MAX_AXIS_VALUES];
    guide_model models[GUIDE_MAX_MODELS];
    guide_hw hw[GUIDE_MAX_HW];
    double eff_c[GUIDE_MAX_EFF];
    double eff_b[GUIDE_MAX_EFF];
};

}  // namespace guide
