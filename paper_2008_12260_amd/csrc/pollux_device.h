// Device-side building blocks shared by the fitness and search kernels:
// 64-lane wavefront exchange through DPP and ds_swizzle, and wave reductions.
// gfx950 only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace px {

constexpr int kWave = 64;

__device__ __forceinline__ int lane_id() { return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)); }

// ---- lane exchange ---------------------------------------------------------
// Every lane receives the value of a partner lane chosen so that six steps
// combine all 64 lanes: quad permutes (partner = lane^1, lane^2), mirror
// within 8 and within 16 lanes (DPP), lane^16 (ds_swizzle in bit mode:
// and 0x1F, or 0, xor 0x10), and lane^32 (ds_bpermute).  All four DPP patterns
// write every lane, so the moves need no previous value.
template <int STEP>
__device__ __forceinline__ int exchange(int v)
{
    if constexpr (STEP == 0) return __builtin_amdgcn_mov_dpp(v, 0xB1, 0xF, 0xF, false);    // quad_perm [1,0,3,2]
    if constexpr (STEP == 1) return __builtin_amdgcn_mov_dpp(v, 0x4E, 0xF, 0xF, false);    // quad_perm [2,3,0,1]
    if constexpr (STEP == 2) return __builtin_amdgcn_mov_dpp(v, 0x141, 0xF, 0xF, false);   // row_half_mirror
    if constexpr (STEP == 3) return __builtin_amdgcn_mov_dpp(v, 0x140, 0xF, 0xF, false);   // row_mirror
    if constexpr (STEP == 4) return __builtin_amdgcn_ds_swizzle(v, 0x401F);                // lane ^ 16
    return __builtin_amdgcn_ds_bpermute((lane_id() ^ 32) << 2, v);                         // lane ^ 32
}

template <int STEP>
__device__ __forceinline__ double exchange(double v)
{
    int lo = __double2loint(v), hi = __double2hiint(v);
    return __hiloint2double(exchange<STEP>(hi), exchange<STEP>(lo));
}

template <int STEP>
__device__ __forceinline__ long long exchange(long long v)
{
    int lo = (int)(v & 0xFFFFFFFFll), hi = (int)(v >> 32);
    return ((long long)exchange<STEP>(hi) << 32) | (long long)(unsigned)exchange<STEP>(lo);
}

// The value lane `src` holds (src the same in every lane).
__device__ __forceinline__ long long wave_broadcast(long long v, int src)
{
    const int lo = __builtin_amdgcn_readlane((int)(v & 0xFFFFFFFFll), src), hi = __builtin_amdgcn_readlane((int)(v >> 32), src);
    return ((long long)hi << 32) | (long long)(unsigned)lo;
}

template <int STEP = 0>
__device__ __forceinline__ long long wave_sum(long long v)
{
    v += exchange<STEP>(v);
    if constexpr (STEP < 5) return wave_sum<STEP + 1>(v);
    return v;
}

// 32-bit reductions: the four DPP steps are folded into the arithmetic
// instruction itself (one VALU instruction per step).
#define PX_DPP_STEPS(OP, v)                                                                              \
    asm("s_nop 1\n\t"                                                                                     \
        OP " %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"                     \
        OP " %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"                     \
        OP " %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"                         \
        OP " %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf"                                             \
        : "+v"(v))

__device__ __forceinline__ int wave_sum(int v)
{
    PX_DPP_STEPS("v_add_u32_dpp", v);
    v += exchange<4>(v);
    v += exchange<5>(v);
    return v;
}

__device__ __forceinline__ int wave_min(int v)
{
    PX_DPP_STEPS("v_min_i32_dpp", v);
    int o = exchange<4>(v);
    v = o < v ? o : v;
    o = exchange<5>(v);
    return o < v ? o : v;
}

__device__ __forceinline__ unsigned wave_min(unsigned v)
{
    PX_DPP_STEPS("v_min_u32_dpp", v);
    unsigned o = (unsigned)exchange<4>((int)v);
    v = o < v ? o : v;
    o = (unsigned)exchange<5>((int)v);
    return o < v ? o : v;
}

__device__ __forceinline__ unsigned wave_max(unsigned v)
{
    PX_DPP_STEPS("v_max_u32_dpp", v);
    unsigned o = (unsigned)exchange<4>((int)v);
    v = o > v ? o : v;
    o = (unsigned)exchange<5>((int)v);
    return o > v ? o : v;
}

}  // namespace px
