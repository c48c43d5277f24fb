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

// `into` with the value of lane LANE replaced by `value` (the same in every lane: it is read from a scalar register).
template <int LANE>
__device__ __forceinline__ int write_lane(int into, int value)
{
    asm("v_writelane_b32 %0, %1, %2" : "+v"(into) : "s"(value), "n"(LANE));
    return into;
}

// The same for a lane number 0 .. 7 that is a constant once the caller's loop is unrolled.
__device__ __forceinline__ int write_lane8(int into, int value, int lane)
{
    switch (lane) {
    case 0: return write_lane<0>(into, value);
    case 1: return write_lane<1>(into, value);
    case 2: return write_lane<2>(into, value);
    case 3: return write_lane<3>(into, value);
    case 4: return write_lane<4>(into, value);
    case 5: return write_lane<5>(into, value);
    case 6: return write_lane<6>(into, value);
    default: return write_lane<7>(into, value);
    }
}

// Every lane receives the value of the lane eight below it in its row of 16 lanes; the lower eight lanes of a row receive 0.
__device__ __forceinline__ int row16_up8(int v) { return __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, true); }   // row_shr:8

template <int STEP = 0>
__device__ __forceinline__ long long wave_sum(long long v)
{
    v += exchange<STEP>(v);
    if constexpr (STEP < 5) return wave_sum<STEP + 1>(v);
    return v;
}

// 32-bit reductions: every step is folded into the arithmetic instruction itself (one VALU
// instruction per step).  Four steps inside each row of 16 lanes leave the row's result in all of
// its lanes; row_bcast:15 then combines rows 0 and 1 into row 1 and rows 2 and 3 into row 3, and
// row_bcast:31 combines those into row 3, so lane 63 holds the result of the wavefront, which is
// read back as a scalar (the same value for every lane).
#define PX_DPP_REDUCE(OP, v)                                                                             \
    asm("s_nop 1\n\t"                                                                                     \
        OP " %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"                     \
        OP " %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"                     \
        OP " %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"                         \
        OP " %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"                              \
        OP " %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\ts_nop 1\n\t"                            \
        OP " %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf"                                           \
        : "+v"(v))

// The same four steps alone: every lane receives the result of its own row of 16 lanes.
#define PX_DPP_ROW_REDUCE(OP, v)                                                                         \
    asm("s_nop 1\n\t"                                                                                     \
        OP " %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"                     \
        OP " %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"                     \
        OP " %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"                         \
        OP " %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf"                                             \
        : "+v"(v))

// Sum over the lane's row of 16 lanes, returned in every lane of that row.
__device__ __forceinline__ int row16_sum(int v)
{
    PX_DPP_ROW_REDUCE("v_add_u32_dpp", v);
    return v;
}

// Smallest value in the lane's row of 16 lanes, returned in every lane of that row.
__device__ __forceinline__ unsigned row16_min(unsigned v)
{
    PX_DPP_ROW_REDUCE("v_min_u32_dpp", v);
    return v;
}

__device__ __forceinline__ int wave_sum(int v)
{
    PX_DPP_REDUCE("v_add_u32_dpp", v);
    return __builtin_amdgcn_readlane(v, 63);
}

__device__ __forceinline__ int wave_min(int v)
{
    PX_DPP_REDUCE("v_min_i32_dpp", v);
    return __builtin_amdgcn_readlane(v, 63);
}

__device__ __forceinline__ unsigned wave_min(unsigned v)
{
    PX_DPP_REDUCE("v_min_u32_dpp", v);
    return (unsigned)__builtin_amdgcn_readlane((int)v, 63);
}

__device__ __forceinline__ unsigned wave_max(unsigned v)
{
    PX_DPP_REDUCE("v_max_u32_dpp", v);
    return (unsigned)__builtin_amdgcn_readlane((int)v, 63);
}

}  // namespace px
