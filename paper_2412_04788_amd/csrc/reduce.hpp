// Wave / LDS reduction helpers shared by the selection and sampled-space kernels.
#pragma once

#include "common.hpp"

namespace guide {

constexpr uint64_t kNone = ~0ull;

// Order-preserving map double -> u64 (-0 folded into +0; NaN never reaches here).
__device__ inline uint64_t key_of(double x) {
    const uint64_t b = (uint64_t)__double_as_longlong(x + 0.0);
    return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
}
__device__ inline double value_of(uint64_t k) {
    const uint64_t b = (k >> 63) ? (k & 0x7FFFFFFFFFFFFFFFull) : ~k;
    return __longlong_as_double((long long)b);
}

struct Pair {
    uint64_t key, idx;
};
__device__ inline bool less_than(const Pair &a, const Pair &b) {
    return a.key < b.key || (a.key == b.key && a.idx < b.idx);
}
__device__ inline Pair pair_min(const Pair &a, const Pair &b) { return less_than(b, a) ? b : a; }

__device__ inline Pair wave_min(Pair p) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        Pair o;
        o.key = __shfl_xor(p.key, off, kWave);
        o.idx = __shfl_xor(p.idx, off, kWave);
        p = pair_min(p, o);
    }
    return p;
}


// Per-wave LDS slots holding the least (key, row) pair per group.  A wave's LDS
// operations execute in program order for all its lanes, so one update is: read
// the key slot, atomic-min the key, read it back; lanes that hold the new
// minimum reset the row slot when the minimum strictly improved and then
// atomic-min their row into it.  Every lane of the wave must call this together
// (inactive lanes pass ok = false).
__device__ inline void slot_update(uint64_t *s_key, uint64_t *s_idx, uint32_t g, bool ok, const Pair &p) {
    uint64_t prev = kNone, cur = kNone;
    if (ok) {
        prev = __hip_atomic_load(&s_key[g], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        __hip_atomic_fetch_min(&s_key[g], p.key, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    __builtin_amdgcn_wave_barrier();
    if (ok) cur = __hip_atomic_load(&s_key[g], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    const bool winner = ok && p.key == cur;
    if (winner && cur < prev) __hip_atomic_store(&s_idx[g], kNone, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    __builtin_amdgcn_wave_barrier();
    if (winner) __hip_atomic_fetch_min(&s_idx[g], p.idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    __builtin_amdgcn_wave_barrier();
}

}  // namespace guide
