// Wavefront-wide reductions shared by the kernels that rank expert logits and reduce dot products
// (Sec. 3.1: softmax denominators, gate-weight sums, top-k maxima; M = 1 decode: row . vector products).
#pragma once

#include "common.h"

namespace remoe {

// One DPP lane permute of a float (no LDS traffic): dpp_ctrl as in the ISA's DPP_CTRL encoding.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
#else
    return v;
#endif
}

__device__ __forceinline__ float read_lane(float v, int l)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
#else
    (void)l;
    return v;
#endif
}

// Sum over the 64 lanes, the same value in every lane, always in the same order (results repeat bit
// for bit): within quads, half rows and rows of 16 by DPP permutes, then the four row sums by lane
// reads.
__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]
    v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]
    v += dpp_move<0x141>(v);   // row_half_mirror
    v += dpp_move<0x140>(v);   // row_mirror
    return (read_lane(v, 0) + read_lane(v, 16)) + (read_lane(v, 32) + read_lane(v, 48));
}

// Maximum over the 64 lanes, the same value in every lane.
__device__ __forceinline__ float wave_max(float v)
{
    v = fmaxf(v, dpp_move<0xB1>(v));
    v = fmaxf(v, dpp_move<0x4E>(v));
    v = fmaxf(v, dpp_move<0x141>(v));
    v = fmaxf(v, dpp_move<0x140>(v));
    return fmaxf(fmaxf(read_lane(v, 0), read_lane(v, 16)), fmaxf(read_lane(v, 32), read_lane(v, 48)));
}

// Minimum of an unsigned value over the 64 lanes, the same value in every lane.
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v)
{
#if defined(__HIP_DEVICE_COMPILE__)
#define REMOE_DPP_U32(x, ctrl) ((uint32_t)__builtin_amdgcn_update_dpp(0, (int)(x), ctrl, 0xF, 0xF, true))
    uint32_t o;
    o = REMOE_DPP_U32(v, 0xB1); v = o < v ? o : v;
    o = REMOE_DPP_U32(v, 0x4E); v = o < v ? o : v;
    o = REMOE_DPP_U32(v, 0x141); v = o < v ? o : v;
    o = REMOE_DPP_U32(v, 0x140); v = o < v ? o : v;
#undef REMOE_DPP_U32
    const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)v, 0), b = (uint32_t)__builtin_amdgcn_readlane((int)v, 16);
    const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)v, 32), d = (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
    const uint32_t ab = a < b ? a : b, cd = c < d ? c : d;
    return ab < cd ? ab : cd;
#else
    return v;
#endif
}

}  // namespace remoe
