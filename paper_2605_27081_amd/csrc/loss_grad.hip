// Gradient of ReMoE's router regularisers with respect to the router logits, and the gate gradient
// it induces (the backward half of the gate-only fine-tuning step of Sec. 4.1; losses of Sec. 4.2-4.4).
//
// Per sequence L = c0 L_Reuse + c1 L_Trust + c2 L_Smooth + c3 L_Lag + c4 L_WS (Eq. 3, 6), P_t =
// softmax(z_t).  With g = dL/dP_t (each entry of P_t taken as a free variable):
//
//   L_Reuse :  -1 / ((rho + 1e-8) (T-1) K) on the entries of E_{t-1} (t >= 2): the previous routed
//              set is a stop-gradient target (Eq. 2, 7)
//   L_Trust :  (ln P_t - ln P_t^ref + 1) / T                                            (Eq. 4-5)
//   SymKL(P, R) w.r.t. P:  phi(P, R) = (ln P - ln R + 1 - R / P) / 2, and the same with the roles
//              exchanged w.r.t. R, so every partner of P_t contributes phi(P_t, partner)   (Eq. 8)
//   L_Smooth:  partners t-1 and t+1, / (T-1)          (no stop-gradient, Sec. 4.4)     (Eq. 9)
//   L_Lag   :  partners t-d and t+d for d in D, / ((T-1) |D|)                           (Eq. 10)
//   L_WS    :  -(ln Pbar_b + 1) / (n W) for the steps of complete windows               (Eq. 11-12)
//
// and dL/dz_t = P_t (g - <P_t, g>).  Entries with P_t[k] = 0 get 0.  The gate gradient of a router
// without bias (Sec. 3.1) is dL/dW_r = sum_t dz_t x_t^T.
//
// loss_window_log_kernel: ln of the window means (fp64), one wavefront per window.
// loss_grad_kernel: one wavefront per step, lane l holding experts l and l + 64; fp64 arithmetic
//   from the fp32 probabilities, terms added in the order listed above; fp32 result.
// gate_grad_partial_kernel: dz^T x on the fp32 matrix cores (v_mfma_f32_32x32x2_f32).  Both operands
//   are read from global memory directly in the instruction's operand layout (lane (i, k) takes
//   dz[t0 + k][e0 + i] and x[t0 + k][h0 + i]: 32 consecutive floats per half wavefront), so no LDS
//   staging is needed.  A wavefront owns all experts x 64 hidden columns for a range of tokens; the
//   four wavefronts of a workgroup add their accumulators through LDS, each workgroup writes its
//   partial tile, and gate_grad_reduce_kernel adds the partial tiles in a fixed order.
#include "common.h"

namespace remoe {

namespace {

constexpr int LG_WAVES = 4;
constexpr int LG_CHUNKS = 64;          // chunks of steps per sequence (loss_grad_kernel grid.x)

__device__ __forceinline__ double wsum64(double v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const unsigned long long b = (unsigned long long)__double_as_longlong(v);
        const unsigned lo = __shfl_xor((unsigned)(b & 0xFFFFFFFFull), off, 64);
        const unsigned hi = __shfl_xor((unsigned)(b >> 32), off, 64);
        v += __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
    }
    return v;
}

struct GradArgs {
    const float *probs, *probs_ref;
    const int32_t *idx;
    const double *loss_values;          // [S, 6]: rho at [s, 0]
    int64_t T;
    int N, K, n_lags, window;
    int lags[8];
    double coef[5];
    double *logbar;                     // [S, n_win, N]
    float *dlogits;                     // [S, T, N]
};

__global__ __launch_bounds__(LG_WAVES * 64) void loss_window_log_kernel(const GradArgs a)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t s = blockIdx.y;
    const int64_t n_win = a.T / a.window;
    const int64_t b = (int64_t)blockIdx.x * LG_WAVES + wave;
    if (b >= n_win) return;
    const int N = a.N;
    const float *P = a.probs + s * a.T * N;
    double m0 = 0.0, m1 = 0.0;
    for (int j = 0; j < a.window; ++j) {
        const int64_t t = b * a.window + j;
        if (lane < N) m0 += (double)P[t * N + lane];
        if (lane + 64 < N) m1 += (double)P[t * N + lane + 64];
    }
    m0 /= (double)a.window;
    m1 /= (double)a.window;
    double *o = a.logbar + (s * n_win + b) * N;
    if (lane < N) o[lane] = log(m0);
    if (lane + 64 < N) o[lane + 64] = log(m1);
}

// (ln p - ln r + 1 - r / p) / 2 for p > 0
__device__ __forceinline__ double phi(double p, double lp, double r) { return 0.5 * (lp - log(r) + 1.0 - r / p); }

__global__ __launch_bounds__(LG_WAVES * 64) void loss_grad_kernel(const GradArgs a)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t s = blockIdx.y;
    const int N = a.N, K = a.K;
    const int64_t T = a.T;
    const float *P = a.probs + s * T * N, *Q = a.probs_ref + s * T * N;
    const int32_t *E = a.idx + s * T * K;
    const int64_t n_win = T / a.window;
    const double rho = a.loss_values[s * 6];
    const double c_reuse = T > 1 ? a.coef[0] * -1.0 / ((rho + 1e-8) * (double)(T - 1) * (double)K) : 0.0;
    const bool has0 = lane < N, has1 = lane + 64 < N;

    const int64_t per = (T + gridDim.x - 1) / gridDim.x;
    const int64_t t_lo = blockIdx.x * per, t_hi = (t_lo + per < T) ? t_lo + per : T;
    for (int64_t t = t_lo + wave; t < t_hi; t += LG_WAVES) {
        const double p0 = has0 ? (double)P[t * N + lane] : 0.0;
        const double p1 = has1 ? (double)P[t * N + lane + 64] : 0.0;
        double g0 = 0.0, g1 = 0.0;
        if (t >= 1)
            for (int j = 0; j < K; ++j) {
                const int e = E[(t - 1) * K + j];
                if (e == lane) g0 += c_reuse;
                if (e == lane + 64) g1 += c_reuse;
            }
        const int64_t b = t / a.window;
        const double *lb = a.logbar + (s * n_win + (b < n_win ? b : 0)) * N;
#define LG_ENTRY(p, g, col)                                                                          \
    if (p > 0.0) {                                                                                   \
        const double lp = log(p);                                                                    \
        g += a.coef[1] * (lp - log((double)Q[t * N + (col)]) + 1.0) / (double)T;                     \
        if (T > 1) {                                                                                 \
            double sm = 0.0, lg = 0.0;                                                               \
            if (t >= 1) sm += phi(p, lp, (double)P[(t - 1) * N + (col)]);                            \
            if (t + 1 < T) sm += phi(p, lp, (double)P[(t + 1) * N + (col)]);                         \
            for (int i = 0; i < a.n_lags; ++i) {                                                     \
                const int d = a.lags[i];                                                             \
                if (t - d >= 0) lg += phi(p, lp, (double)P[(t - d) * N + (col)]);                    \
                if (t + d < T) lg += phi(p, lp, (double)P[(t + d) * N + (col)]);                     \
            }                                                                                        \
            g += a.coef[2] * sm / (double)(T - 1);                                                   \
            if (a.n_lags > 0) g += a.coef[3] * lg / ((double)(T - 1) * (double)a.n_lags);            \
        }                                                                                            \
        if (b < n_win) g += a.coef[4] * -(lb[(col)] + 1.0) / ((double)n_win * (double)a.window);     \
    } else {                                                                                         \
        g = 0.0;                                                                                     \
    }
        if (has0) { LG_ENTRY(p0, g0, lane) }
        if (has1) { LG_ENTRY(p1, g1, lane + 64) }
#undef LG_ENTRY
        const double dot = wsum64(p0 * g0 + p1 * g1);
        float *o = a.dlogits + (s * T + t) * N;
        if (has0) o[lane] = (float)(p0 * (g0 - dot));
        if (has1) o[lane + 64] = (float)(p1 * (g1 - dot));
    }
}

// ---- gate gradient ---------------------------------------------------------------------------------

constexpr int GG_NH = 2;                // 32-column tiles of hidden per wavefront
constexpr int GG_COLS = GG_NH * 32;     // hidden columns per workgroup
constexpr int GG_MAX_NE = 4;            // 32-row tiles of experts (N <= 128)
constexpr int GG_WAVES = 4;

struct GateArgs {
    const float *dz;                    // [T, N]
    const void *x;                      // [T, H] bf16 or fp32
    int64_t T;
    int N, H, chunks;
    float *partial;                     // [chunks, N, H]
    float *dw;                          // [N, H]
};

// loads through pointers known to point to device memory (global, not flat, address space)
__device__ __forceinline__ float load_global_f32(const void *p) { return *(const __attribute__((address_space(1))) float *)p; }
template <class XT> __device__ __forceinline__ float x_as_float(const XT *p);
template <> __device__ __forceinline__ float x_as_float<float>(const float *p) { return load_global_f32(p); }
template <> __device__ __forceinline__ float x_as_float<bf16_t>(const bf16_t *p)
{
    return __uint_as_float((uint32_t)(*(const __attribute__((address_space(1))) bf16_t *)p) << 16);
}

template <class XT, int NE>
__global__ __launch_bounds__(GG_WAVES * 64) void gate_grad_partial_kernel(const GateArgs a)
{
    __shared__ float red[NE * GG_NH * 16 * 64];   // one wavefront's accumulators at a time
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane & 31, lh = lane >> 5;
    const int h0 = blockIdx.x * GG_COLS;
    const int chunk = blockIdx.y;
    const int N = a.N, H = a.H;
    const XT *x = static_cast<const XT *>(a.x);

    floatx16_t acc[NE][GG_NH];
#pragma unroll
    for (int e = 0; e < NE; ++e)
#pragma unroll
        for (int n = 0; n < GG_NH; ++n)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[e][n][r] = 0.f;

    // this wavefront's tokens: an even number per wavefront so that token pairs never straddle
    const int64_t per_wg = (a.T + a.chunks - 1) / a.chunks;
    const int64_t per_wave = ((per_wg + GG_WAVES - 1) / GG_WAVES + 1) & ~(int64_t)1;
    const int64_t wg_lo = chunk * per_wg, wg_hi = (wg_lo + per_wg < a.T) ? wg_lo + per_wg : a.T;
    int64_t t_lo = wg_lo + wave * per_wave, t_hi = t_lo + per_wave;
    if (t_hi > wg_hi) t_hi = wg_hi;

    // GG_UN token pairs per pass.  The operand loads of the next pass are issued before the MFMAs of
    // the current one (two register sets), so that a wavefront alone on its SIMD still overlaps load
    // latency with matrix-core work.  Loads are unconditional (clamped indices) and masked by a
    // multiplication: a conditional load is a branch, and behind every branch the compiler waits for
    // all loads in flight.  (What a masked load reads is other tokens' or experts' data of the same call.)
    constexpr int GG_UN = 2;
    const int n_tok = (int)(t_hi > t_lo ? t_hi - t_lo : 0);
    const int n_pairs = (n_tok + 1) >> 1;
    const char *dz_w = reinterpret_cast<const char *>(a.dz + t_lo * N);
    const char *x_w = reinterpret_cast<const char *>(x + t_lo * H + h0);
    uint32_t dz_col[NE];
    float col_live[NE];
#pragma unroll
    for (int e = 0; e < NE; ++e) {
        const int col = e * 32 + li;
        dz_col[e] = (uint32_t)(col < N ? col : N - 1) * 4u;
        col_live[e] = col < N ? 1.0f : 0.f;
    }
#define GG_LOAD(av, bv, first_pair)                                                                      \
    _Pragma("unroll") for (int u = 0; u < GG_UN; ++u) {                                                  \
        const int t_ = 2 * ((first_pair) + u) + lh;      /* k index of the instruction = which token of the pair */ \
        const int tc_ = t_ < n_tok ? t_ : n_tok - 1;                                                     \
        _Pragma("unroll") for (int e = 0; e < NE; ++e)                                                   \
            av[u][e] = load_global_f32(dz_w + (uint32_t)(tc_ * N) * 4u + dz_col[e]);                     \
        _Pragma("unroll") for (int n = 0; n < GG_NH; ++n)                                                \
            bv[u][n] = x_as_float<XT>(reinterpret_cast<const XT *>(x_w + (uint32_t)(tc_ * H + n * 32 + li) * (uint32_t)sizeof(XT))); \
    }
    // the masks are applied here, not where the values are requested: a use right behind a load is a wait
#define GG_MFMA(av, bv, first_pair)                                                                      \
    _Pragma("unroll") for (int u = 0; u < GG_UN; ++u) {                                                  \
        const float live_ = (2 * ((first_pair) + u) + lh < n_tok) ? 1.0f : 0.f;                          \
        _Pragma("unroll") for (int e = 0; e < NE; ++e)                                                   \
            _Pragma("unroll") for (int n = 0; n < GG_NH; ++n)                                            \
                acc[e][n] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u][e] * col_live[e], bv[u][n] * live_, acc[e][n], 0, 0, 0); \
    }
    if (n_tok > 0) {
        float avA[GG_UN][NE], bvA[GG_UN][GG_NH], avB[GG_UN][NE], bvB[GG_UN][GG_NH];
        GG_LOAD(avA, bvA, 0)
#pragma unroll 1
        for (int i = 0; i < n_pairs; i += 2 * GG_UN) {
            __builtin_amdgcn_sched_barrier(0);
            GG_LOAD(avB, bvB, i + GG_UN)                 // past the end: clamped and masked to zero
            __builtin_amdgcn_sched_barrier(0);
            GG_MFMA(avA, bvA, i)
            __builtin_amdgcn_sched_barrier(0);
            GG_LOAD(avA, bvA, i + 2 * GG_UN)
            __builtin_amdgcn_sched_barrier(0);
            GG_MFMA(avB, bvB, i + GG_UN)
        }
    }
#undef GG_LOAD
#undef GG_MFMA

    // add the four wavefronts' accumulators in wavefront order (one at a time through one LDS buffer:
    // a small LDS footprint lets several workgroups share a compute unit and hide each other's load
    // latency), then write the workgroup's tile
    for (int w = 1; w < GG_WAVES; ++w) {
        if (wave == w) {
#pragma unroll
            for (int e = 0; e < NE; ++e)
#pragma unroll
                for (int n = 0; n < GG_NH; ++n)
#pragma unroll
                    for (int r = 0; r < 16; ++r) red[((e * GG_NH + n) * 16 + r) * 64 + lane] = acc[e][n][r];
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int e = 0; e < NE; ++e)
#pragma unroll
                for (int n = 0; n < GG_NH; ++n)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[e][n][r] += red[((e * GG_NH + n) * 16 + r) * 64 + lane];
        }
        __syncthreads();
    }
    if (wave == 0) {
        float *out = a.partial + (int64_t)chunk * N * H;
#pragma unroll
        for (int e = 0; e < NE; ++e)
#pragma unroll
            for (int n = 0; n < GG_NH; ++n)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = e * 32 + (r >> 2) * 8 + lh * 4 + (r & 3);     // expert
                    if (row < N) out[(int64_t)row * H + h0 + n * 32 + li] = acc[e][n][r];
                }
    }
}

__global__ void gate_grad_reduce_kernel(const GateArgs a)
{
    const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t total = (int64_t)a.N * a.H;
    if (q >= total) return;
    float v = 0.f;
    for (int c = 0; c < a.chunks; ++c) v += a.partial[(int64_t)c * total + q];
    a.dw[q] = v;
}

int gate_grad_chunks(int64_t T, int H)
{
    // about four workgroups per compute unit at the widest hidden sizes, at least 64 tokens each
    int64_t c = 1024 / (H / GG_COLS > 0 ? H / GG_COLS : 1);
    if (c < 1) c = 1;
    if (c > 64) c = 64;
    while (c > 1 && T / c < 64) c >>= 1;
    return (int)c;
}

}  // namespace

size_t loss_backward_workspace_bytes(int64_t S, int64_t T, int N, int window)
{
    const int64_t n_win = window > 0 ? T / window : 0;
    return align_up(sizeof(double) * (size_t)(S * n_win * N) + 8, 256);
}

remoe_status launch_loss_backward(const float *probs, const float *probs_ref, const int32_t *idx, int64_t S, int64_t T,
                                  int N, int K, const int32_t *lags, int n_lags, int window, const double *coef,
                                  const double *loss_values, float *dlogits, void *workspace, hipStream_t stream)
{
    if (S == 0 || T == 0) return REMOE_OK;
    if (S > 65535) return fail(REMOE_E_UNSUPPORTED, "remoe_loss_backward handles at most 65535 sequences per call (got %lld)", (long long)S);
    GradArgs a;
    a.probs = probs; a.probs_ref = probs_ref; a.idx = idx; a.loss_values = loss_values;
    a.T = T; a.N = N; a.K = K; a.n_lags = n_lags; a.window = window;
    for (int i = 0; i < 8; ++i) a.lags[i] = i < n_lags ? lags[i] : 0;
    for (int i = 0; i < 5; ++i) a.coef[i] = coef[i];
    a.logbar = static_cast<double *>(workspace);
    a.dlogits = dlogits;
    const int64_t n_win = T / window;
    if (n_win > 0) {
        if (ceil_div(n_win, LG_WAVES) > 0x7FFFFFFF) return fail(REMOE_E_UNSUPPORTED, "too many windows");
        hipLaunchKernelGGL(loss_window_log_kernel, dim3((unsigned)ceil_div(n_win, LG_WAVES), (unsigned)S), dim3(LG_WAVES * 64), 0,
                           stream, a);
    }
    const int chunks = (int)(T < LG_CHUNKS * LG_WAVES ? ceil_div(T, LG_WAVES) : LG_CHUNKS);
    hipLaunchKernelGGL(loss_grad_kernel, dim3((unsigned)chunks, (unsigned)S), dim3(LG_WAVES * 64), 0, stream, a);
    return check_hip(hipGetLastError(), "loss gradient kernels launch");
}

size_t gate_grad_workspace_bytes(int64_t T, int N, int H)
{
    return align_up(sizeof(float) * (size_t)gate_grad_chunks(T, H) * (size_t)N * (size_t)H, 256);
}

remoe_status launch_gate_grad(const float *dz, const void *x, int x_dtype, int64_t T, int N, int H, float *dw, void *workspace,
                              hipStream_t stream)
{
    if (H % GG_COLS != 0) return fail(REMOE_E_UNSUPPORTED, "remoe_gate_grad needs hidden %% %d == 0 (got %d)", GG_COLS, H);
    if (N > GG_MAX_NE * 32) return fail(REMOE_E_UNSUPPORTED, "remoe_gate_grad handles at most %d experts", GG_MAX_NE * 32);
    GateArgs a;
    a.dz = dz; a.x = x; a.T = T; a.N = N; a.H = H;
    a.chunks = gate_grad_chunks(T, H);
    a.partial = static_cast<float *>(workspace);
    a.dw = dw;
    const dim3 grid((unsigned)(H / GG_COLS), (unsigned)a.chunks), block(GG_WAVES * 64);
    const int ne = (N + 31) / 32;
#define GG_LAUNCH(XT)                                                                                              \
    switch (ne) {                                                                                                  \
    case 1: hipLaunchKernelGGL((gate_grad_partial_kernel<XT, 1>), grid, block, 0, stream, a); break;               \
    case 2: hipLaunchKernelGGL((gate_grad_partial_kernel<XT, 2>), grid, block, 0, stream, a); break;               \
    case 3: hipLaunchKernelGGL((gate_grad_partial_kernel<XT, 3>), grid, block, 0, stream, a); break;               \
    default: hipLaunchKernelGGL((gate_grad_partial_kernel<XT, 4>), grid, block, 0, stream, a); break;              \
    }
    if (x_dtype == REMOE_BF16) { GG_LAUNCH(bf16_t) } else { GG_LAUNCH(float) }
#undef GG_LAUNCH
    const int64_t total = (int64_t)N * H;
    hipLaunchKernelGGL(gate_grad_reduce_kernel, dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, stream, a);
    return check_hip(hipGetLastError(), "gate gradient kernels launch");
}

}  // namespace remoe
