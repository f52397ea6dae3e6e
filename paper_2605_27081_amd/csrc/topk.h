// Wavefront-shuffle top-k and softmax over one token's expert logits (Sec. 3.1:
// P_t = Softmax(logits), E_t = Top-K(P_t)).  Shared by the batched router and the M = 1 decode kernel.
//
// Lane l owns the logits of experts l and l + 64 (-inf where the expert does not exist).  K (+1)
// rounds of a 6-step butterfly argmax over (logit, -id) select the experts in descending-logit
// order with ties to the lower id; softmax is taken over all N experts with the maximum subtracted.
#pragma once

#include "common.h"

namespace remoe {

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

struct TopKResult {
    int expert;     // lanes j < K: id of the j-th selected expert
    float weight;   // lanes j < K: its gate weight (renormalised over the K when asked)
    float margin;   // all lanes: logit_(K) - logit_(K+1), +inf when K == N
    float e0, e1;   // this lane's exp(logit - max) for experts lane and lane + 64 (0 where absent)
    float den;      // all lanes: sum of exp(logit - max) over the N experts
};

__device__ __forceinline__ TopKResult wave_topk_softmax(float v0, float v1, int N, int K, int renorm, int lane)
{
    const float NEG_INF = -__builtin_inff();
    const int rounds = (K < N) ? K + 1 : K;
    float c0 = v0, c1 = v1;
    float my_v = 0.f, zmax = 0.f, zk = 0.f, zk1 = 0.f;
    TopKResult res;
    res.expert = 0;
#pragma unroll 1
    for (int j = 0; j < rounds; ++j) {
        const bool pick1 = c1 > c0;
        float bv = pick1 ? c1 : c0;
        int be = pick1 ? lane + 64 : lane;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const float ov = __shfl_xor(bv, off, 64);
            const int oe = __shfl_xor(be, off, 64);
            if (ov > bv || (ov == bv && oe < be)) { bv = ov; be = oe; }
        }
        if (j < K) {
            if (lane == j) { my_v = bv; res.expert = be; }
            if (j == 0) zmax = bv;
            zk = bv;
            if (be == lane) c0 = NEG_INF;
            if (be == lane + 64) c1 = NEG_INF;
        } else {
            zk1 = bv;
        }
    }
    res.e0 = (lane < N) ? expf(v0 - zmax) : 0.f;
    res.e1 = (lane + 64 < N) ? expf(v1 - zmax) : 0.f;
    res.den = wave_sum(res.e0 + res.e1);
    const float my_p = (lane < K) ? expf(my_v - zmax) : 0.f;
    res.weight = my_p / res.den;
    if (renorm) {
        const float sel = wave_sum(my_p);
        res.weight = my_p / sel;
    }
    res.margin = (K < N) ? zk - zk1 : __builtin_inff();
    return res;
}

}  // namespace remoe
