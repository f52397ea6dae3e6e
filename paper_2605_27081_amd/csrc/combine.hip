// Weighted combine: y[t] = sum_{j<K} out_j(t) + s_t * shared(t), summed in fp32.
//
// The routed part is the sum of the token's K rows, each weighted by its gate weight P_t[e]
// (Sec. 3.1), found through the pair -> slot map of the permute step and taken in routing order
// (descending logit).  The weights come from pair_w in (token, j) order; where pair_w is NULL the
// down-projection kernel has already applied them (the fp32 path) and the rows are summed as they
// are.  The shared
// expert's row (always active, outside P_t) is added last, scaled by s_t = sigmoid(ws_scale . x[t])
// when the layer gates its shared expert.  One workgroup per token; the sum order is fixed, so the
// result is deterministic.
#include "common.h"

namespace remoe {

namespace {

template <typename ET> struct Vec;

template <> struct Vec<float> {
    static constexpr int N = 4;
    __device__ static __forceinline__ void load(const float *p, float *o)
    {
        const float4 v = *reinterpret_cast<const float4 *>(p);
        o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
    }
    __device__ static __forceinline__ void store(float *p, const float *o)
    {
        *reinterpret_cast<float4 *>(p) = make_float4(o[0], o[1], o[2], o[3]);
    }
};

template <> struct Vec<bf16_t> {
    static constexpr int N = 8;
    __device__ static __forceinline__ void load(const bf16_t *p, float *o)
    {
        const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));   // every row is read once
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            o[2 * i] = __uint_as_float(w[i] << 16);
            o[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
    __device__ static __forceinline__ void store(bf16_t *p, const float *o)
    {
        u32x4_t v;
        v.x = pack_bf16x2(o[0], o[1]);
        v.y = pack_bf16x2(o[2], o[3]);
        v.z = pack_bf16x2(o[4], o[5]);
        v.w = pack_bf16x2(o[6], o[7]);
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t *>(p));
    }
};

template <typename ET>
__global__ __launch_bounds__(256) void combine_kernel(const ET *__restrict__ rows,
                                                      const int32_t *__restrict__ pair_slot,
                                                      const float *__restrict__ pair_w, int K, int H, int64_t shared_row0, int has_shared,
                                                      const ET *__restrict__ x,
                                                      const float *__restrict__ ws_scale,
                                                      ET *__restrict__ y)
{
    constexpr int V = Vec<ET>::N;
    __shared__ float red[4];
    const int64_t t = blockIdx.x;
    const int tid = threadIdx.x;
    float s = 1.0f;
    if (has_shared && ws_scale) {
        float part = 0.f;
        for (int c = tid; c < H / V; c += 256) {
            float xv[V];
            Vec<ET>::load(x + t * H + c * V, xv);
#pragma unroll
            for (int i = 0; i < V; ++i) part = fmaf(xv[i], ws_scale[c * V + i], part);
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) part += __shfl_xor(part, off, 64);
        if ((tid & 63) == 0) red[tid >> 6] = part;
        __syncthreads();
        const float dot = (red[0] + red[1]) + (red[2] + red[3]);
        s = 1.0f / (1.0f + expf(-dot));
    }
    int slot[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) slot[j] = (j < K) ? pair_slot[t * K + j] : 0;
    float wj[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) wj[j] = (j < K && pair_w) ? pair_w[t * K + j] : 1.0f;
    for (int c = tid; c < H / V; c += 256) {
        float acc[V];
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (j < K) {
                float v[V];
                Vec<ET>::load(rows + (int64_t)slot[j] * H + c * V, v);
#pragma unroll
                for (int i = 0; i < V; ++i) acc[i] = fmaf(wj[j], v[i], acc[i]);
            }
        }
        if (has_shared) {
            float v[V];
            Vec<ET>::load(rows + (shared_row0 + t) * H + c * V, v);
#pragma unroll
            for (int i = 0; i < V; ++i) acc[i] = fmaf(s, v[i], acc[i]);
        }
        Vec<ET>::store(y + t * H + c * V, acc);
    }
}

}  // namespace

remoe_status launch_combine(int dtype, const void *rows, const int32_t *pair_slot, const float *pair_w, int64_t T, int K,
                            int H, int64_t shared_row0, int has_shared, const void *x,
                            const float *ws_scale, void *y, hipStream_t stream)
{
    if (T == 0) return REMOE_OK;
    const dim3 grid((unsigned)T), block(256);
    if (dtype == REMOE_F32)
        hipLaunchKernelGGL(combine_kernel<float>, grid, block, 0, stream, static_cast<const float *>(rows),
                           pair_slot, pair_w, K, H, shared_row0, has_shared, static_cast<const float *>(x),
                           ws_scale, static_cast<float *>(y));
    else
        hipLaunchKernelGGL(combine_kernel<bf16_t>, grid, block, 0, stream,
                           static_cast<const bf16_t *>(rows), pair_slot, pair_w, K, H, shared_row0, has_shared,
                           static_cast<const bf16_t *>(x), ws_scale, static_cast<bf16_t *>(y));
    return check_hip(hipGetLastError(), "combine launch");
}

}  // namespace remoe
