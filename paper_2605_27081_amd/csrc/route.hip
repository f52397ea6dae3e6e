// Router kernel: fp32 logits on the fp32 matrix cores, then a wavefront-shuffle top-k and softmax.
//
// Computes the paper's routing step (Sec. 3.1): P_t = Softmax(h_t^T theta_gate), E_t = Top-K(P_t).
// One workgroup (4 wavefronts) owns 128 tokens and all N_r <= 128 experts, so every token's full
// logit row ends in one wavefront: 32 tokens x (NT*32) experts per wavefront as NT accumulators of
// v_mfma_f32_32x32x2_f32.  The logits are parked in LDS and each token is then ranked by its
// wavefront: every lane owns experts {lane, lane+64}, and K+1 rounds of a 6-step butterfly argmax
// over (logit, -id) produce the ids in descending-logit order with ties to the lower id.
#include "common.h"
#include "topk.h"

namespace remoe {

namespace {

constexpr int RT_BM = 128;  // tokens per workgroup
constexpr int RT_BK = 32;   // reduction slice per LDS stage (fp32 elements)

// LDS tiles hold rows of 32 floats = 8 chunks of 16 bytes; chunk c of row r lives in row slot
// r ^ ((r >> 3) & 1) at chunk position c ^ (r & 7), so that the rows a wavefront reads at once
// spread over all banks whether 8 or 16 lanes are served per cycle.
__device__ __forceinline__ int swz(int r, int c)
{
    return (r ^ ((r >> 3) & 1)) * RT_BK + ((c ^ (r & 7)) << 2);
}

template <typename XT> struct XLoad;

template <> struct XLoad<float> {
    // 128 rows x 8 chunks(4 floats): 4 chunks per thread
    floatx4_t v[4];
    __device__ __forceinline__ void load(const float *x, int64_t t0, int64_t T, int H, int k0, int tid)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int q = tid + 256 * i, r = q >> 3, c = q & 7;
            int64_t t = t0 + r;
            if (t >= T) t = T - 1;
            v[i] = *reinterpret_cast<const floatx4_t *>(x + t * H + k0 + c * 4);
        }
    }
    __device__ __forceinline__ void store(float *as, int tid) const
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int q = tid + 256 * i, r = q >> 3, c = q & 7;
            *reinterpret_cast<floatx4_t *>(as + swz(r, c)) = v[i];
        }
    }
};

template <> struct XLoad<bf16_t> {
    // 128 rows x 4 chunks(8 bf16): 2 chunks per thread, each widened to two fp32 chunks
    u32x4_t v[2];
    __device__ __forceinline__ void load(const bf16_t *x, int64_t t0, int64_t T, int H, int k0, int tid)
    {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            int q = tid + 256 * i, r = q >> 2, c = q & 3;
            int64_t t = t0 + r;
            if (t >= T) t = T - 1;
            v[i] = *reinterpret_cast<const u32x4_t *>(x + t * H + k0 + c * 8);
        }
    }
    __device__ __forceinline__ void store(float *as, int tid) const
    {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            int q = tid + 256 * i, r = q >> 2, c = q & 3;
            const u32x4_t w = v[i];
            floatx4_t lo, hi;
            lo.x = __uint_as_float(w.x << 16); lo.y = __uint_as_float(w.x & 0xFFFF0000u);
            lo.z = __uint_as_float(w.y << 16); lo.w = __uint_as_float(w.y & 0xFFFF0000u);
            hi.x = __uint_as_float(w.z << 16); hi.y = __uint_as_float(w.z & 0xFFFF0000u);
            hi.z = __uint_as_float(w.w << 16); hi.w = __uint_as_float(w.w & 0xFFFF0000u);
            *reinterpret_cast<floatx4_t *>(as + swz(r, 2 * c)) = lo;
            *reinterpret_cast<floatx4_t *>(as + swz(r, 2 * c + 1)) = hi;
        }
    }
};

template <int NT, typename XT>
__global__ __launch_bounds__(256) void route_kernel(const XT *__restrict__ x, int64_t T, int H,
                                                    const float *__restrict__ wr, int N, int K,
                                                    int renorm, int32_t *__restrict__ out_idx,
                                                    float *__restrict__ out_w,
                                                    float *__restrict__ out_margin,
                                                    float *__restrict__ out_probs)
{
    constexpr int NE = NT * 32;
    constexpr int A_FLOATS = RT_BM * RT_BK;
    constexpr int B_FLOATS = NE * RT_BK;
    constexpr int TILE_FLOATS = 2 * A_FLOATS + 2 * B_FLOATS;
    constexpr int LOGIT_FLOATS = RT_BM * NE;
    constexpr int SMEM_FLOATS = TILE_FLOATS > LOGIT_FLOATS ? TILE_FLOATS : LOGIT_FLOATS;
    __shared__ __attribute__((aligned(16))) float smem[SMEM_FLOATS];
    float *As = smem;
    float *Bs = smem + 2 * A_FLOATS;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int li = lane & 31;   // row / column inside a 32x32 MFMA tile
    const int lh = lane >> 5;   // which k of the pair this lane feeds
    const int64_t t0 = (int64_t)blockIdx.x * RT_BM;

    floatx16_t acc[NT];
#pragma unroll
    for (int n = 0; n < NT; ++n)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[n][r] = 0.f;

    XLoad<XT> xa;
    floatx4_t bv[NT];
#define RT_LOAD_B(k0)                                                                         \
    _Pragma("unroll") for (int i = 0; i < NT; ++i) {                                           \
        const int q_ = tid + 256 * i, r_ = q_ >> 3, c_ = q_ & 7;                              \
        const floatx4_t zero_ = {0.f, 0.f, 0.f, 0.f};                                          \
        bv[i] = (r_ < N) ? *reinterpret_cast<const floatx4_t *>(wr + (int64_t)r_ * H + (k0) + c_ * 4) \
                         : zero_;                                                             \
    }
#define RT_STORE_B(bs)                                                                        \
    _Pragma("unroll") for (int i = 0; i < NT; ++i) {                                           \
        const int q_ = tid + 256 * i, r_ = q_ >> 3, c_ = q_ & 7;                              \
        *reinterpret_cast<floatx4_t *>((bs) + swz(r_, c_)) = bv[i];                            \
    }

    const int nk = H / RT_BK;
    xa.load(x, t0, T, H, 0, tid);
    RT_LOAD_B(0)
    xa.store(As, tid);
    RT_STORE_B(Bs)
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) {
            xa.load(x, t0, T, H, (kt + 1) * RT_BK, tid);
            RT_LOAD_B((kt + 1) * RT_BK)
        }
        const float *as = As + cur * A_FLOATS;
        const float *bs = Bs + cur * B_FLOATS;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            // this lane's four k values of the group: 8q + 4*lh + {0..3}
            const floatx4_t a4 = *reinterpret_cast<const floatx4_t *>(as + swz(wave * 32 + li, 2 * q + lh));
            floatx4_t b4[NT];
#pragma unroll
            for (int n = 0; n < NT; ++n)
                b4[n] = *reinterpret_cast<const floatx4_t *>(bs + swz(n * 32 + li, 2 * q + lh));
#pragma unroll
            for (int s = 0; s < 4; ++s) {
#pragma unroll
                for (int n = 0; n < NT; ++n)
                    acc[n] = __builtin_amdgcn_mfma_f32_32x32x2f32(a4[s], b4[n][s], acc[n], 0, 0, 0);
            }
        }
        if (kt + 1 < nk) {
            xa.store(As + (cur ^ 1) * A_FLOATS, tid);
            RT_STORE_B(Bs + (cur ^ 1) * B_FLOATS)
        }
        __syncthreads();
    }

    // park the logits: row = token inside the workgroup, column = expert
    float *Ls = smem;
#pragma unroll
    for (int n = 0; n < NT; ++n)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = wave * 32 + (r >> 2) * 8 + lh * 4 + (r & 3);
            Ls[row * NE + n * 32 + li] = acc[n][r];
        }
    __syncthreads();

    const float NEG_INF = -__builtin_inff();
#pragma unroll 1
    for (int tl = 0; tl < 32; ++tl) {
        const int64_t t = t0 + wave * 32 + tl;
        if (t >= T) break;
        const float *L = Ls + (wave * 32 + tl) * NE;
        const float v0 = (lane < N) ? L[lane] : NEG_INF;
        float v1 = NEG_INF;
        if (NE > 64) v1 = (lane + 64 < N) ? L[lane + 64] : NEG_INF;
        const TopKResult r = wave_topk_softmax(v0, v1, N, K, renorm, lane);
        if (lane < K) {
            out_idx[t * K + lane] = r.expert;
            out_w[t * K + lane] = r.weight;
        }
        if (out_margin && lane == 0) out_margin[t] = r.margin;
        if (out_probs) {
            if (lane < N) out_probs[t * N + lane] = r.e0 / r.den;
            if (lane + 64 < N) out_probs[t * N + lane + 64] = r.e1 / r.den;
        }
    }
}

template <typename XT>
remoe_status launch_typed(const XT *x, int64_t T, int H, const float *wr, int N, int K, int renorm,
                          int32_t *out_idx, float *out_w, float *out_margin, float *out_probs,
                          hipStream_t stream)
{
    const dim3 grid((unsigned)ceil_div(T, RT_BM)), block(256);
    if (N <= 32)
        hipLaunchKernelGGL((route_kernel<1, XT>), grid, block, 0, stream, x, T, H, wr, N, K, renorm,
                           out_idx, out_w, out_margin, out_probs);
    else if (N <= 64)
        hipLaunchKernelGGL((route_kernel<2, XT>), grid, block, 0, stream, x, T, H, wr, N, K, renorm,
                           out_idx, out_w, out_margin, out_probs);
    else
        hipLaunchKernelGGL((route_kernel<4, XT>), grid, block, 0, stream, x, T, H, wr, N, K, renorm,
                           out_idx, out_w, out_margin, out_probs);
    return check_hip(hipGetLastError(), "route_kernel launch");
}

}  // namespace

remoe_status launch_route(const void *x, int x_dtype, int64_t T, int H, const float *w_router,
                          int N, int K, int renorm, int32_t *out_idx, float *out_w,
                          float *out_margin, float *out_probs, hipStream_t stream)
{
    if (T == 0) return REMOE_OK;
    if (x_dtype == REMOE_F32)
        return launch_typed<float>(static_cast<const float *>(x), T, H, w_router, N, K, renorm,
                                   out_idx, out_w, out_margin, out_probs, stream);
    return launch_typed<bf16_t>(static_cast<const bf16_t *>(x), T, H, w_router, N, K, renorm,
                                out_idx, out_w, out_margin, out_probs, stream);
}

}  // namespace remoe
