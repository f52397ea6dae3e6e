// Router kernel: fp32-accurate logits on the matrix cores, then a lane-per-token top-k and softmax.
//
// Computes the paper's routing step (Sec. 3.1): P_t = Softmax(h_t^T theta_gate), E_t = Top-K(P_t).
// One workgroup (4 wavefronts) owns 128 tokens and all N_r <= 128 experts, so every token's full
// logit row ends in one workgroup: 32 tokens x (NT*32) experts per wavefront as NT accumulators.
//
// Logits.  The gate weights are fp32 and the logits must carry fp32 accuracy (near ties decide
// which experts run).  For fp32 hidden states the products run on v_mfma_f32_32x32x2_f32.  For bf16
// hidden states every x is already exact in bf16, and each fp32 weight is split on the fly into three
// bf16 pieces w = hi + mid + lo (each the round-to-nearest of what the previous ones left, 24+
// significand bits in all), so x*hi, x*mid and x*lo are exact fp32 products and three
// v_mfma_f32_32x32x16_bf16 with fp32 accumulation replace sixteen fp32 MFMA steps.
//
// Top-k.  The logits are parked in LDS, one padded row per token.  Two neighbouring lanes share a
// token, each scanning half of its experts in ascending id and keeping the 9 largest (K <= 8, plus
// the runner-up for the margin) by insertion into a sorted register list; strict comparisons keep
// the lower id first among equal logits.  The halves are merged through a lane swap, the softmax
// denominator is summed the same way, and the pair writes ids and weights of its token.
#include "common.h"

namespace remoe {

namespace {

constexpr int RT_BM = 128;   // tokens per workgroup
constexpr int RT_BK = 32;    // reduction slice per LDS stage (elements)
constexpr int RT_LIST = 9;   // sorted candidates kept per lane: MAX top_k + 1

// ---- fp32 path: LDS tiles hold rows of 32 floats = 8 chunks of 16 bytes; chunk c of row r lives in
// row slot r ^ ((r >> 3) & 1) at chunk position c ^ (r & 7), so that the rows a wavefront reads at
// once spread over all banks whether 8 or 16 lanes are served per cycle.
__device__ __forceinline__ int swz_f32(int r, int c)
{
    return (r ^ ((r >> 3) & 1)) * RT_BK + ((c ^ (r & 7)) << 2);
}

// ---- bf16 path: rows of 32 bf16 = 4 chunks of 16 bytes; chunk c of row r sits at chunk position
// c ^ ((r >> 2) & 3), which makes 16 consecutive rows of one logical chunk cover all 16 slots of a
// 256-byte period.  Returns the offset in 16-byte units.
__device__ __forceinline__ int swz_bf16(int r, int c) { return r * 4 + (c ^ ((r >> 2) & 3)); }

// round-to-nearest-even bf16 pieces of two neighbouring fp32 weights: w = hi + mid + lo up to 2^-24
// relative, each piece packed the way the LDS tiles hold it (first weight in the low half); three
// packed conversions (v_cvt_pk_bf16_f32) for the pair
__device__ __forceinline__ void split3_pair(float w0, float w1, uint32_t &hi, uint32_t &mid, uint32_t &lo)
{
    hi = pack_bf16x2(w0, w1);
    const float r0 = w0 - __uint_as_float(hi << 16), r1 = w1 - __uint_as_float(hi & 0xFFFF0000u);
    mid = pack_bf16x2(r0, r1);
    const float q0 = r0 - __uint_as_float(mid << 16), q1 = r1 - __uint_as_float(mid & 0xFFFF0000u);
    lo = pack_bf16x2(q0, q1);
}

// Logit rows in LDS: experts [0, NE/2) then 4 floats of padding, experts [NE/2, NE), 4 more.  With a
// row stride of NE + 8 floats the 16-byte reads of 8 tokens x 2 halves fall into 16 different slots.
template <int NE> struct LogitLayout {
    static constexpr int HALF = NE / 2;
    static constexpr int STRIDE = NE + 8;
    __device__ static __forceinline__ int at(int row, int col) { return row * STRIDE + col + (col >= HALF ? 4 : 0); }
};

// ---- logits of fp32 hidden states: 2-stage LDS pipeline, v_mfma_f32_32x32x2_f32
template <int NT>
__device__ __forceinline__ void logits_f32(const float *__restrict__ x, int64_t t0, int64_t T, int H,
                                           const float *__restrict__ wr, int N, float *smem,
                                           floatx16_t (&acc)[NT], int tid)
{
    constexpr int NE = NT * 32;
    constexpr int A_FLOATS = RT_BM * RT_BK;
    constexpr int B_FLOATS = NE * RT_BK;
    float *As = smem;
    float *Bs = smem + 2 * A_FLOATS;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;

    floatx4_t av[4], bv[NT];
#define RT_LOAD_F32(k0)                                                                        \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                             \
        const int q_ = tid + 256 * i, r_ = q_ >> 3, c_ = q_ & 7;                               \
        int64_t t_ = t0 + r_;                                                                  \
        if (t_ >= T) t_ = T - 1;                                                               \
        av[i] = *reinterpret_cast<const floatx4_t *>(x + t_ * H + (k0) + c_ * 4);              \
    }                                                                                          \
    _Pragma("unroll") for (int i = 0; i < NT; ++i) {                                            \
        const int q_ = tid + 256 * i, r_ = q_ >> 3, c_ = q_ & 7;                               \
        const floatx4_t zero_ = {0.f, 0.f, 0.f, 0.f};                                           \
        bv[i] = (r_ < N) ? *reinterpret_cast<const floatx4_t *>(wr + (int64_t)r_ * H + (k0) + c_ * 4) \
                         : zero_;                                                              \
    }
#define RT_STORE_F32(as, bs)                                                                   \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                             \
        const int q_ = tid + 256 * i, r_ = q_ >> 3, c_ = q_ & 7;                               \
        *reinterpret_cast<floatx4_t *>((as) + swz_f32(r_, c_)) = av[i];                         \
    }                                                                                          \
    _Pragma("unroll") for (int i = 0; i < NT; ++i) {                                            \
        const int q_ = tid + 256 * i, r_ = q_ >> 3, c_ = q_ & 7;                               \
        *reinterpret_cast<floatx4_t *>((bs) + swz_f32(r_, c_)) = bv[i];                         \
    }

    const int nk = H / RT_BK;
    RT_LOAD_F32(0)
    RT_STORE_F32(As, Bs)
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) { RT_LOAD_F32((kt + 1) * RT_BK) }
        const float *as = As + cur * A_FLOATS;
        const float *bs = Bs + cur * B_FLOATS;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            // this lane's four k values of the group: 8q + 4*lh + {0..3}
            const floatx4_t a4 = *reinterpret_cast<const floatx4_t *>(as + swz_f32(wave * 32 + li, 2 * q + lh));
            floatx4_t b4[NT];
#pragma unroll
            for (int n = 0; n < NT; ++n)
                b4[n] = *reinterpret_cast<const floatx4_t *>(bs + swz_f32(n * 32 + li, 2 * q + lh));
#pragma unroll
            for (int s = 0; s < 4; ++s) {
#pragma unroll
                for (int n = 0; n < NT; ++n)
                    acc[n] = __builtin_amdgcn_mfma_f32_32x32x2f32(a4[s], b4[n][s], acc[n], 0, 0, 0);
            }
        }
        if (kt + 1 < nk) { RT_STORE_F32(As + (cur ^ 1) * A_FLOATS, Bs + (cur ^ 1) * B_FLOATS) }
        __syncthreads();
    }
#undef RT_LOAD_F32
#undef RT_STORE_F32
}

// ---- logits of bf16 hidden states: x as stored, weights as three bf16 pieces, v_mfma_f32_32x32x16_bf16
template <int NT>
__device__ __forceinline__ void logits_bf16(const bf16_t *__restrict__ x, int64_t t0, int64_t T, int H,
                                            const float *__restrict__ wr, int N, float *smem,
                                            floatx16_t (&acc)[NT], int tid)
{
    constexpr int NE = NT * 32;
    constexpr int A_U4 = RT_BM * 4;          // 16-byte units of one x stage
    constexpr int P_U4 = NE * 4;             // ... of one weight piece
    constexpr int STAGE_U4 = A_U4 + 3 * P_U4;
    u32x4_t *base = reinterpret_cast<u32x4_t *>(smem);
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;

    u32x4_t xv[2];
    floatx4_t wv[NT];
#define RT_LOAD_BF16(k0)                                                                       \
    _Pragma("unroll") for (int i = 0; i < 2; ++i) {                                             \
        const int q_ = tid + 256 * i, r_ = q_ >> 2, c_ = q_ & 3;                               \
        int64_t t_ = t0 + r_;                                                                  \
        if (t_ >= T) t_ = T - 1;                                                               \
        xv[i] = *reinterpret_cast<const u32x4_t *>(x + t_ * H + (k0) + c_ * 8);                \
    }                                                                                          \
    _Pragma("unroll") for (int i = 0; i < NT; ++i) {                                            \
        const int q_ = tid + 256 * i, r_ = q_ >> 3, c_ = q_ & 7;                               \
        const floatx4_t zero_ = {0.f, 0.f, 0.f, 0.f};                                           \
        wv[i] = (r_ < N) ? *reinterpret_cast<const floatx4_t *>(wr + (int64_t)r_ * H + (k0) + c_ * 4) \
                         : zero_;                                                              \
    }
    // a thread holds 4 consecutive k of one weight row: half a 16-byte chunk of each piece
#define RT_STORE_BF16(st)                                                                      \
    _Pragma("unroll") for (int i = 0; i < 2; ++i) {                                             \
        const int q_ = tid + 256 * i, r_ = q_ >> 2, c_ = q_ & 3;                               \
        (st)[swz_bf16(r_, c_)] = xv[i];                                                        \
    }                                                                                          \
    _Pragma("unroll") for (int i = 0; i < NT; ++i) {                                            \
        const int q_ = tid + 256 * i, r_ = q_ >> 3, c_ = q_ & 7;                               \
        uint32_t h_[2], m_[2], l_[2];                                                          \
        split3_pair(wv[i][0], wv[i][1], h_[0], m_[0], l_[0]);                                  \
        split3_pair(wv[i][2], wv[i][3], h_[1], m_[1], l_[1]);                                  \
        uint2 *dst_ = reinterpret_cast<uint2 *>((st) + A_U4 + swz_bf16(r_, c_ >> 1)) + (c_ & 1); \
        dst_[0] = make_uint2(h_[0], h_[1]);                                                    \
        dst_[2 * P_U4] = make_uint2(m_[0], m_[1]);                                              \
        dst_[4 * P_U4] = make_uint2(l_[0], l_[1]);                                              \
    }

    const int nk = H / RT_BK;
    RT_LOAD_BF16(0)
    RT_STORE_BF16(base)
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) { RT_LOAD_BF16((kt + 1) * RT_BK) }
        const u32x4_t *st = base + cur * STAGE_U4;
        if (NT == 4) {
            // 128 experts: wavefront w takes expert tile w for all four token tiles, so a k-step reads
            // 4 token fragments + 3 weight pieces from LDS (7 KB) instead of 1 + 12 (13 KB); the sums
            // are the same, element by element and in the same order
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                bf16x8_t a8[NT], w8[3];
#pragma unroll
                for (int m = 0; m < NT; ++m)
                    a8[m] = *reinterpret_cast<const bf16x8_t *>(&st[swz_bf16(m * 32 + li, 2 * ks + lh)]);
#pragma unroll
                for (int pc = 0; pc < 3; ++pc)
                    w8[pc] = *reinterpret_cast<const bf16x8_t *>(
                        &st[A_U4 + pc * P_U4 + swz_bf16(wave * 32 + li, 2 * ks + lh)]);
#pragma unroll
                for (int pc = 0; pc < 3; ++pc)
#pragma unroll
                    for (int m = 0; m < NT; ++m)
                        acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a8[m], w8[pc], acc[m], 0, 0, 0);
            }
        } else
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            // this lane's eight k values of the step: 16 ks + 8 lh + {0..7} = chunk 2 ks + lh
            const bf16x8_t a8 = *reinterpret_cast<const bf16x8_t *>(&st[swz_bf16(wave * 32 + li, 2 * ks + lh)]);
            bf16x8_t b8[NT][3];
#pragma unroll
            for (int n = 0; n < NT; ++n)
#pragma unroll
                for (int pc = 0; pc < 3; ++pc)
                    b8[n][pc] = *reinterpret_cast<const bf16x8_t *>(
                        &st[A_U4 + pc * P_U4 + swz_bf16(n * 32 + li, 2 * ks + lh)]);
#pragma unroll
            for (int pc = 0; pc < 3; ++pc)
#pragma unroll
                for (int n = 0; n < NT; ++n)
                    acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a8, b8[n][pc], acc[n], 0, 0, 0);
        }
        if (kt + 1 < nk) { RT_STORE_BF16(base + (cur ^ 1) * STAGE_U4) }
        __syncthreads();
    }
#undef RT_LOAD_BF16
#undef RT_STORE_BF16
}

template <int NT, typename XT> struct SmemFloats {
    static constexpr int NE = NT * 32;
    static constexpr int TILES = sizeof(XT) == 4 ? 2 * (RT_BM * RT_BK + NE * RT_BK)            // fp32 tiles
                                                 : 2 * (RT_BM * 4 + 3 * NE * 4) * 4;           // bf16 tiles
    static constexpr int LOGITS = RT_BM * LogitLayout<NE>::STRIDE;
    static constexpr int VALUE = TILES > LOGITS ? TILES : LOGITS;
};

// (v, id) goes into the descending list if it beats an entry; what falls off the end is dropped
#define RT_INSERT(v_in, id_in, BEATS)                                                          \
    {                                                                                          \
        float v_ = (v_in);                                                                     \
        int id_ = (id_in);                                                                     \
        _Pragma("unroll") for (int s = 0; s < RT_LIST; ++s) {                                   \
            const bool gt_ = BEATS(v_, id_, val[s], idx[s]);                                   \
            const float tv_ = gt_ ? val[s] : v_;                                               \
            const int ti_ = gt_ ? idx[s] : id_;                                                \
            val[s] = gt_ ? v_ : val[s];                                                        \
            idx[s] = gt_ ? id_ : idx[s];                                                       \
            v_ = tv_;                                                                          \
            id_ = ti_;                                                                         \
        }                                                                                      \
    }
#define RT_BEATS_SCAN(v, i, lv, li_) ((v) > (lv))                                  /* ids arrive ascending */
#define RT_BEATS_ANY(v, i, lv, li_) ((v) > (lv) || ((v) == (lv) && (i) < (li_)))   /* any order */

template <int NT, typename XT>
__global__ __launch_bounds__(256) void route_kernel(const XT *__restrict__ x, int64_t T, int H,
                                                    const float *__restrict__ wr, int N, int K,
                                                    int renorm, int32_t *__restrict__ out_idx,
                                                    float *__restrict__ out_w,
                                                    float *__restrict__ out_margin,
                                                    float *__restrict__ out_probs)
{
    constexpr int NE = NT * 32;
    typedef LogitLayout<NE> LL;
    __shared__ __attribute__((aligned(16))) float smem[SmemFloats<NT, XT>::VALUE];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int li = lane & 31;   // row / column inside a 32x32 MFMA tile
    const int lh = lane >> 5;
    const int64_t t0 = (int64_t)blockIdx.x * RT_BM;

    floatx16_t acc[NT];
#pragma unroll
    for (int n = 0; n < NT; ++n)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[n][r] = 0.f;

    if (sizeof(XT) == 4)
        logits_f32<NT>(reinterpret_cast<const float *>(x), t0, T, H, wr, N, smem, acc, tid);
    else
        logits_bf16<NT>(reinterpret_cast<const bf16_t *>(x), t0, T, H, wr, N, smem, acc, tid);

    // park the logits (the tile stages are idle after the last barrier of the loop)
    float *Ls = smem;
#pragma unroll
    for (int n = 0; n < NT; ++n)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            // (bf16 hidden states, 128 experts: accumulator n is token tile n of expert tile `wave`)
            const bool by_expert = sizeof(XT) == 2 && NT == 4;
            const int row = (by_expert ? n : wave) * 32 + (r >> 2) * 8 + lh * 4 + (r & 3);
            Ls[LL::at(row, (by_expert ? wave : n) * 32 + li)] = acc[n][r];
        }
    __syncthreads();

    // ---- top-k: lanes 2j and 2j+1 take token j of the workgroup, one half of the experts each
    const float NEG_INF = -__builtin_inff();
    const int tl = tid >> 1, half = tid & 1;
    const int64_t t = t0 + tl;
    const int e_base = half * LL::HALF;
    const float *row = Ls + tl * LL::STRIDE + half * (LL::HALF + 4);
    float val[RT_LIST];
    int idx[RT_LIST];
#pragma unroll
    for (int s = 0; s < RT_LIST; ++s) { val[s] = NEG_INF; idx[s] = 0x7FFFFFFF; }
#pragma unroll 2
    for (int e4 = 0; e4 < LL::HALF; e4 += 4) {
        const floatx4_t v4 = *reinterpret_cast<const floatx4_t *>(row + e4);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int e = e_base + e4 + j;
            RT_INSERT((e < N) ? v4[j] : NEG_INF, e, RT_BEATS_SCAN)
        }
    }
    // merge with the neighbour's list (both lanes end with the same merged list)
    {
        float pv[RT_LIST];
        int pi[RT_LIST];
#pragma unroll
        for (int s = 0; s < RT_LIST; ++s) {
            pv[s] = swap_with_neighbour(val[s]);
            pi[s] = __float_as_int(swap_with_neighbour(__int_as_float(idx[s])));
        }
#pragma unroll
        for (int s = 0; s < RT_LIST; ++s) RT_INSERT(pv[s], pi[s], RT_BEATS_ANY)
    }
    // softmax denominator over all N experts, maximum subtracted
    const float zmax = val[0];
    float part = 0.f;
    for (int e4 = 0; e4 < LL::HALF; e4 += 4) {
        const floatx4_t v4 = *reinterpret_cast<const floatx4_t *>(row + e4);
#pragma unroll
        for (int j = 0; j < 4; ++j) part += (e_base + e4 + j < N) ? __expf(v4[j] - zmax) : 0.f;
    }
    const float den = part + swap_with_neighbour(part);

    if (t < T) {
        float pk[RT_LIST - 1];
        float sel = 0.f;
#pragma unroll
        for (int j = 0; j < RT_LIST - 1; ++j) {
            pk[j] = (j < K) ? __expf(val[j] - zmax) : 0.f;
            sel += pk[j];
        }
        const float inv = 1.0f / (renorm ? sel : den);
        // the even lane writes the ids, the odd lane the weights
#pragma unroll
        for (int j = 0; j < RT_LIST - 1; ++j) {
            if (j < K) {
                if (half == 0) out_idx[t * K + j] = idx[j];
                else out_w[t * K + j] = pk[j] * inv;
            }
        }
        if (out_margin && half == 0) {
            float zk = val[0], zk1 = val[1];
#pragma unroll
            for (int j = 1; j < RT_LIST - 1; ++j)
                if (j < K) { zk = val[j]; zk1 = val[j + 1]; }
            out_margin[t] = (K < N) ? zk - zk1 : __builtin_inff();
        }
        if (out_probs) {
            const float rden = 1.0f / den;
            for (int e = 0; e < LL::HALF; ++e)
                if (e_base + e < N) out_probs[t * N + e_base + e] = __expf(row[e] - zmax) * rden;
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
