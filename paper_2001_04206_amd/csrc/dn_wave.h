// Wave-level reductions shared by the kernels of this library (64-lane wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>

namespace dn {

// Wave-wide reductions with data-parallel-primitive moves (no LDS traffic): butterflies inside
// each row of 16 lanes, then the row totals are carried across rows; lane 63 ends up with the
// result, which is broadcast through a scalar register.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_move(float v, float identity)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, identity),
                                                                 __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xf,
                                                                 false));
}

__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_move<0xB1, 0xf>(v, 0.f);    // quad_perm [1,0,3,2]
    v += dpp_move<0x4E, 0xf>(v, 0.f);    // quad_perm [2,3,0,1]
    v += dpp_move<0x141, 0xf>(v, 0.f);   // row_half_mirror
    v += dpp_move<0x140, 0xf>(v, 0.f);   // row_mirror: every lane of a row holds the row's sum
    v += dpp_move<0x142, 0xa>(v, 0.f);   // row_bcast:15 into rows 1 and 3
    v += dpp_move<0x143, 0xc>(v, 0.f);   // row_bcast:31 into rows 2 and 3
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

__device__ __forceinline__ float wave_max(float v)
{
    const float ninf = -INFINITY;
    v = fmaxf(v, dpp_move<0xB1, 0xf>(v, ninf));
    v = fmaxf(v, dpp_move<0x4E, 0xf>(v, ninf));
    v = fmaxf(v, dpp_move<0x141, 0xf>(v, ninf));
    v = fmaxf(v, dpp_move<0x140, 0xf>(v, ninf));
    v = fmaxf(v, dpp_move<0x142, 0xa>(v, ninf));
    v = fmaxf(v, dpp_move<0x143, 0xc>(v, ninf));
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// Completes this wave's device-scope stores before it signals another workgroup.
// Data that crosses workgroups is written with relaxed device-scope atomic stores, which the
// hardware performs as write-through stores to the level all workgroups of the device share.  A
// wave's memory counter reaches zero only when every store it has issued has been acknowledged
// from that level (the compiler's own code for a device-scope release leans on the same fact), so
// after this call -- and a workgroup barrier, when another wave does the signalling -- a flag or
// counter written with a device-scope atomic is observed only after the data.  The workgroup-scope
// release fence keeps the compiler from sinking stores below the wait.  Unlike a device-scope
// release fence this does not write back the L2, which such stores never leave dirty.
__device__ __forceinline__ void drain_device_scope_stores()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);   // vmcnt, expcnt, lgkmcnt = 0
}

// Sum over each aligned group of 16 lanes (a DPP row); every lane of the group gets it.
__device__ __forceinline__ float row16_sum(float v)
{
    v += dpp_move<0xB1, 0xf>(v, 0.f);
    v += dpp_move<0x4E, 0xf>(v, 0.f);
    v += dpp_move<0x141, 0xf>(v, 0.f);
    v += dpp_move<0x140, 0xf>(v, 0.f);
    return v;
}

}  // namespace dn
