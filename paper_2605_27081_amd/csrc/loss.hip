// Forward values of ReMoE's router regularisers on a batch of routing distributions (Sec. 4.2-4.4):
//
//   m_t      = (1/K) sum_{k in E_{t-1}} P_t[k]                               (Eq. 2, reuse mass)
//   rho      = mean_{t>=2} m_t,   L_Reuse = -log(rho + 1e-8)                 (Eq. 7)
//   L_Trust  = mean_t KL(P_t || P_t^ref)                                     (Eq. 4-5)
//   L_Smooth = mean_{t>=2} SymKL(P_t, P_{t-1})                               (Eq. 8-9)
//   L_Lag    = mean_{t>=2} (1/|D|) sum_{d in D, t-d>=1} SymKL(P_t, P_{t-d})  (Eq. 10)
//   L_WS     = mean_b H(mean of the W distributions of window b)             (Eq. 11-12)
//
// per sequence.  The inputs are the fp32 probabilities the router kernel writes; everything here is
// computed in fp64 (the work is ~7 N logarithms per step, nothing next to the expert GEMMs), with
// SymKL(P,Q) = (1/2) sum_k (P[k] - Q[k]) (ln P[k] - ln Q[k]).
//
// loss_partial_kernel: grid (chunk, sequence); a workgroup's 4 wavefronts take the steps (and the
// windows) of its chunk in turn, lane l holding experts l and l + 64; per-wavefront fp64 sums are
// combined in wavefront order and written to the workspace.  loss_final_kernel adds the chunks of
// a sequence in chunk order and applies the normalisations, so results repeat bit for bit.
#include "common.h"

namespace remoe {

namespace {

constexpr int LS_CHUNKS = 16;           // chunks of steps (and of windows) per sequence
constexpr int LS_WAVES = 4;
constexpr int LS_TERMS = 5;             // sum m_t, sum KL, sum SymKL adjacent, sum lag term, sum window entropy

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

struct Row {
    double p0, p1, l0, l1;              // probabilities of experts lane, lane + 64 and their logarithms
};

__device__ __forceinline__ Row load_row(const float *__restrict__ base, int64_t t, int N, int lane)
{
    Row r;
    r.p0 = lane < N ? (double)base[t * N + lane] : 0.0;
    r.p1 = lane + 64 < N ? (double)base[t * N + lane + 64] : 0.0;
    r.l0 = r.p0 > 0.0 ? log(r.p0) : 0.0;
    r.l1 = r.p1 > 0.0 ? log(r.p1) : 0.0;
    return r;
}

// this lane's share of KL(a || b): a ln(a / b), 0 where a = 0 (ln b = -inf where b = 0 and a > 0)
__device__ __forceinline__ double kl_part(double a, double la, double b, double lb)
{
    if (!(a > 0.0)) return 0.0;
    return a * (la - (b > 0.0 ? lb : -__builtin_inf()));
}

__device__ __forceinline__ double symkl_part(const Row &a, const Row &b)
{
    return 0.5 * (kl_part(a.p0, a.l0, b.p0, b.l0) + kl_part(b.p0, b.l0, a.p0, a.l0) +
                  kl_part(a.p1, a.l1, b.p1, b.l1) + kl_part(b.p1, b.l1, a.p1, a.l1));
}

struct LossArgs {
    const float *probs, *probs_ref;
    const int32_t *idx;
    int64_t T;
    int N, K, n_lags, window;
    int lags[8];
    double *partial;                    // [S, LS_CHUNKS, LS_TERMS]
    double *out;                        // [S, 6]
};

__global__ __launch_bounds__(LS_WAVES * 64) void loss_partial_kernel(const LossArgs a)
{
    __shared__ double part[LS_WAVES][LS_TERMS];
    const int chunk = blockIdx.x;
    const int64_t s = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int N = a.N, K = a.K;
    const int64_t T = a.T;
    const float *P = a.probs + s * T * N, *Q = a.probs_ref + s * T * N;
    const int32_t *E = a.idx + s * T * K;
    double acc[LS_TERMS] = {0.0, 0.0, 0.0, 0.0, 0.0};

    const int64_t per = (T + LS_CHUNKS - 1) / LS_CHUNKS;
    const int64_t t_lo = chunk * per, t_hi = (t_lo + per < T) ? t_lo + per : T;
    for (int64_t t = t_lo + wave; t < t_hi; t += LS_WAVES) {
        const Row pt = load_row(P, t, N, lane);
        const Row qt = load_row(Q, t, N, lane);
        acc[1] += kl_part(pt.p0, pt.l0, qt.p0, qt.l0) + kl_part(pt.p1, pt.l1, qt.p1, qt.l1);
        if (t >= 1) {
            if (lane < K) acc[0] += (double)P[t * N + E[(t - 1) * K + lane]];
            for (int i = 0; i < a.n_lags; ++i) {
                const int d = a.lags[i];
                if (t - d < 0) continue;
                const double v = symkl_part(pt, load_row(P, t - d, N, lane));
                acc[3] += v;
                if (d == 1) acc[2] += v;
            }
            bool has_unit = false;
            for (int i = 0; i < a.n_lags; ++i) has_unit |= a.lags[i] == 1;
            if (!has_unit) acc[2] += symkl_part(pt, load_row(P, t - 1, N, lane));
        }
    }
    // windows of this chunk
    const int64_t n_win = T / a.window;
    const int64_t wper = (n_win + LS_CHUNKS - 1) / LS_CHUNKS;
    const int64_t b_lo = chunk * wper, b_hi = (b_lo + wper < n_win) ? b_lo + wper : n_win;
    for (int64_t b = b_lo + wave; b < b_hi; b += LS_WAVES) {
        double m0 = 0.0, m1 = 0.0;
        for (int j = 0; j < a.window; ++j) {
            const int64_t t = b * a.window + j;
            if (lane < N) m0 += (double)P[t * N + lane];
            if (lane + 64 < N) m1 += (double)P[t * N + lane + 64];
        }
        m0 /= (double)a.window;
        m1 /= (double)a.window;
        acc[4] -= (m0 > 0.0 ? m0 * log(m0) : 0.0) + (m1 > 0.0 ? m1 * log(m1) : 0.0);
    }
#pragma unroll
    for (int k = 0; k < LS_TERMS; ++k) {
        const double v = wsum64(acc[k]);
        if (lane == 0) part[wave][k] = v;
    }
    __syncthreads();
    if (threadIdx.x < LS_TERMS) {
        double v = 0.0;
        for (int w = 0; w < LS_WAVES; ++w) v += part[w][threadIdx.x];
        a.partial[(s * LS_CHUNKS + chunk) * LS_TERMS + threadIdx.x] = v;
    }
}

__global__ void loss_final_kernel(const LossArgs a, int64_t S)
{
    const int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= S) return;
    double sum[LS_TERMS] = {0.0, 0.0, 0.0, 0.0, 0.0};
    for (int c = 0; c < LS_CHUNKS; ++c)
        for (int k = 0; k < LS_TERMS; ++k) sum[k] += a.partial[(s * LS_CHUNKS + c) * LS_TERMS + k];
    const int64_t T = a.T;
    const double pairs = T > 1 ? (double)(T - 1) : 1.0;
    const int64_t n_win = T / a.window;
    const double rho = T > 1 ? sum[0] / (double)a.K / pairs : 0.0;
    double *o = a.out + s * 6;
    o[0] = rho;
    o[1] = -log(rho + 1e-8);
    o[2] = T > 0 ? sum[1] / (double)T : 0.0;
    o[3] = T > 1 ? sum[2] / pairs : 0.0;
    o[4] = (T > 1 && a.n_lags > 0) ? sum[3] / (double)a.n_lags / pairs : 0.0;
    o[5] = n_win > 0 ? sum[4] / (double)n_win : 0.0;
}

}  // namespace

size_t loss_workspace_bytes(int64_t S) { return align_up(sizeof(double) * (size_t)S * LS_CHUNKS * LS_TERMS, 256); }

remoe_status launch_loss_forward(const float *probs, const float *probs_ref, const int32_t *idx, int64_t S, int64_t T,
                                 int N, int K, const int32_t *lags, int n_lags, int window, double *out, void *workspace,
                                 hipStream_t stream)
{
    if (S == 0) return REMOE_OK;
    if (S > 65535) return fail(REMOE_E_UNSUPPORTED, "remoe_loss_forward handles at most 65535 sequences per call (got %lld)", (long long)S);
    LossArgs a;
    a.probs = probs; a.probs_ref = probs_ref; a.idx = idx;
    a.T = T; a.N = N; a.K = K; a.n_lags = n_lags; a.window = window;
    for (int i = 0; i < 8; ++i) a.lags[i] = i < n_lags ? lags[i] : 0;
    a.partial = static_cast<double *>(workspace);
    a.out = out;
    hipLaunchKernelGGL(loss_partial_kernel, dim3(LS_CHUNKS, (unsigned)S), dim3(LS_WAVES * 64), 0, stream, a);
    hipLaunchKernelGGL(loss_final_kernel, dim3((unsigned)ceil_div(S, 64)), dim3(64), 0, stream, a, S);
    return check_hip(hipGetLastError(), "loss kernels launch");
}

}  // namespace remoe
