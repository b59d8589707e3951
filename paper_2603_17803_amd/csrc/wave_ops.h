// Wave-level primitives on the DPP data path of gfx950 (64-lane wavefronts, rows of 16 lanes).
// None of them touches LDS.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace waveops {

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_or_zero(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xF, false);
}

// Inclusive prefix sum over the 64 lanes of a wave.
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) {
    v += dpp_or_zero<0x111, 0xF>(v);     // row_shr:1
    v += dpp_or_zero<0x112, 0xF>(v);     // row_shr:2
    v += dpp_or_zero<0x114, 0xF>(v);     // row_shr:4
    v += dpp_or_zero<0x118, 0xF>(v);     // row_shr:8   -> scan inside each row of 16
    v += dpp_or_zero<0x142, 0xA>(v);     // row_bcast:15 into rows 1 and 3
    v += dpp_or_zero<0x143, 0xC>(v);     // row_bcast:31 into rows 2 and 3
    return v;
}

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), CTRL, 0xF, 0xF, false));
}

// Maximum / minimum over the wave, returned in every lane.
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_f<0xB1>(v));        // quad_perm [1,0,3,2]
    v = fmaxf(v, dpp_f<0x4E>(v));        // quad_perm [2,3,0,1]
    v = fmaxf(v, dpp_f<0x141>(v));       // row_half_mirror
    v = fmaxf(v, dpp_f<0x140>(v));       // row_mirror -> row maximum in all 16 lanes
    v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), 0x142, 0xA, 0xF, false)));
    v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), 0x143, 0xC, 0xF, false)));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_min(float v) { return -wave_max(-v); }

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_min_u32(uint32_t v) {
    const uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp(-1, (int)v, CTRL, 0xF, 0xF, false);   // old = identity of min
    return min(v, o);
}

// The same exchange for patterns in which every lane has a source (quad_perm, the row mirrors, all rows and banks
// enabled): "zero for a lane without source" never applies, and saying so leaves the instruction free to write a
// register of its own instead of updating a copy of its input in place.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_min_u32_all(uint32_t v) {
    const uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
    return min(v, o);
}

// Minimum over aligned groups of 2^STEPS lanes (STEPS <= 4), valid in every lane of a group.
template <int STEPS>
__device__ __forceinline__ uint32_t lane_group_min(uint32_t v) {
    static_assert(STEPS >= 2 && STEPS <= 4, "inside a row of 16 lanes");
    v = dpp_min_u32_all<0xB1>(v);                   // quad_perm [1,0,3,2]
    v = dpp_min_u32_all<0x4E>(v);                   // quad_perm [2,3,0,1]
    if (STEPS >= 3) v = dpp_min_u32_all<0x141>(v);  // row_half_mirror
    if (STEPS >= 4) v = dpp_min_u32_all<0x140>(v);  // row_mirror
    return v;
}

// Minimum over the first 2^STEPS lanes, valid in every one of them (STEPS <= 4 stays inside a row of
// 16 lanes and is pure DPP; 5 and 6 add two cross-row shuffles).  Lanes that do not take part must
// hold 0xffffffff.
template <int STEPS>
__device__ __forceinline__ uint32_t low_lanes_min(uint32_t v) {
    v = dpp_min_u32<0xB1>(v);                       // quad_perm [1,0,3,2]
    v = dpp_min_u32<0x4E>(v);                       // quad_perm [2,3,0,1]
    if (STEPS >= 3) v = dpp_min_u32<0x141>(v);      // row_half_mirror
    if (STEPS >= 4) v = dpp_min_u32<0x140>(v);      // row_mirror
    if (STEPS >= 5) v = min(v, (uint32_t)__shfl_xor((int)v, 16, 64));
    if (STEPS >= 6) v = min(v, (uint32_t)__shfl_xor((int)v, 32, 64));
    return v;
}

// Minimum over all 64 lanes, returned in every lane.
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
    v = dpp_min_u32<0xB1>(v);
    v = dpp_min_u32<0x4E>(v);
    v = dpp_min_u32<0x141>(v);
    v = dpp_min_u32<0x140>(v);
    v = min(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x142, 0xA, 0xF, false));   // row_bcast:15
    v = min(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x143, 0xC, 0xF, false));   // row_bcast:31
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// Exclusive prefix sum over the wave plus the wave total.
__device__ __forceinline__ uint32_t wave_excl_scan(uint32_t v, uint32_t* total) {
    const uint32_t incl = wave_incl_scan(v);
    *total = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
    return incl - v;
}

}  // namespace waveops
