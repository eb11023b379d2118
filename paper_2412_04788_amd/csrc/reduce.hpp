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

// Cross-lane moves in the vector ALU (data-parallel primitives, no LDS traffic).  A lane whose
// source lane does not exist for the pattern, or whose row is masked out, receives `old`.
// Patterns used: 0xB1 / 0x4E swap neighbours / pairs inside each group of four lanes, 0x141 / 0x140
// mirror each half-row / row of 16 lanes, 0x110 + n shifts a row right by n lanes, 0x142 / 0x143
// broadcast lane 15 of each row to the next row / lane 31 to the upper two rows.
template <int CTRL, int ROW_MASK = 0xf>
__device__ inline uint32_t dpp_u32(uint32_t old, uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)old, (int)v, CTRL, ROW_MASK, 0xf, false);
}
template <int CTRL, int ROW_MASK = 0xf>
__device__ inline uint64_t dpp_keep(uint64_t v) {       // lanes without a source keep their own value
    const uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
    return ((uint64_t)dpp_u32<CTRL, ROW_MASK>(hi, hi) << 32) | dpp_u32<CTRL, ROW_MASK>(lo, lo);
}
template <int CTRL, int ROW_MASK = 0xf>
__device__ inline Pair dpp_keep(const Pair &p) {
    return Pair{dpp_keep<CTRL, ROW_MASK>(p.key), dpp_keep<CTRL, ROW_MASK>(p.idx)};
}
__device__ inline uint64_t read_lane63(uint64_t v) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, kWave - 1);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), kWave - 1);
    return ((uint64_t)hi << 32) | lo;
}
__device__ inline uint64_t min_u64(uint64_t a, uint64_t b) { return b < a ? b : a; }

// Least value of the wave, in every lane.  Every lane of the wave must be active.  Wider values are
// reduced 32 bits at a time, most significant first: lanes that do not hold the minimum so far drop
// out of the next pass (a 32-bit step is one move-and-minimum; a 64-bit compare-and-select is five).
__device__ inline uint32_t wave_min(uint32_t v) {
    uint32_t o;
    o = dpp_u32<0xB1>(v, v); v = o < v ? o : v;
    o = dpp_u32<0x4E>(v, v); v = o < v ? o : v;
    o = dpp_u32<0x141>(v, v); v = o < v ? o : v;
    o = dpp_u32<0x140>(v, v); v = o < v ? o : v;          // every lane holds the minimum of its row
    o = dpp_u32<0x142, 0xa>(v, v); v = o < v ? o : v;
    o = dpp_u32<0x143, 0xc>(v, v); v = o < v ? o : v;     // lane 63 holds the minimum of the wave
    return (uint32_t)__builtin_amdgcn_readlane((int)v, kWave - 1);
}
__device__ inline uint64_t wave_min(uint64_t v) {
    const uint32_t hi = (uint32_t)(v >> 32), lo = (uint32_t)v;
    const uint32_t m_hi = wave_min(hi);
    const uint32_t m_lo = wave_min(hi == m_hi ? lo : 0xFFFFFFFFu);
    return ((uint64_t)m_hi << 32) | m_lo;
}
// Least (key, idx) pair of the wave in lexicographic order.
__device__ inline Pair wave_min(Pair p) {
    const uint64_t m_key = wave_min(p.key);
    const uint64_t m_idx = wave_min(p.key == m_key ? p.idx : kNone);
    return Pair{m_key, m_idx};
}
__device__ inline uint32_t wave_max(uint32_t v) {
    uint32_t o;
    o = dpp_u32<0xB1>(v, v); v = o > v ? o : v;
    o = dpp_u32<0x4E>(v, v); v = o > v ? o : v;
    o = dpp_u32<0x141>(v, v); v = o > v ? o : v;
    o = dpp_u32<0x140>(v, v); v = o > v ? o : v;
    o = dpp_u32<0x142, 0xa>(v, v); v = o > v ? o : v;
    o = dpp_u32<0x143, 0xc>(v, v); v = o > v ? o : v;
    return (uint32_t)__builtin_amdgcn_readlane((int)v, kWave - 1);
}
// Inclusive scans over the lanes of a wave (every lane active).
__device__ inline uint64_t wave_scan_min(uint64_t v) {
    v = min_u64(v, dpp_keep<0x111>(v));
    v = min_u64(v, dpp_keep<0x112>(v));
    v = min_u64(v, dpp_keep<0x114>(v));
    v = min_u64(v, dpp_keep<0x118>(v));
    v = min_u64(v, dpp_keep<0x142, 0xa>(v));
    v = min_u64(v, dpp_keep<0x143, 0xc>(v));
    return v;
}
__device__ inline uint32_t wave_scan_sum(uint32_t v) {
    v += dpp_u32<0x111>(0u, v);
    v += dpp_u32<0x112>(0u, v);
    v += dpp_u32<0x114>(0u, v);
    v += dpp_u32<0x118>(0u, v);
    v += dpp_u32<0x142, 0xa>(0u, v);
    v += dpp_u32<0x143, 0xc>(0u, v);
    return v;
}

// Sum over the lanes of a wave, in every lane (every lane active).
__device__ inline uint32_t wave_sum(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_readlane((int)wave_scan_sum(v), kWave - 1);
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
