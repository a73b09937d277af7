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
