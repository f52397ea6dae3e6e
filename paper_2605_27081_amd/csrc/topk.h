// Wavefront-wide reduction shared by the kernels that rank expert logits (Sec. 3.1: softmax
// denominators, gate-weight sums).
#pragma once

#include "common.h"

namespace remoe {

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

}  // namespace remoe
