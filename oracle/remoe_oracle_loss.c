/*
 * CPU oracle, third file: the forward value of ReMoE's router regularisers for one batch of
 * routing distributions.
 *
 * TEST INFRASTRUCTURE ONLY (see remoe_oracle.c).  fp64 throughout, from the fp32 probabilities the
 * GPU reads; every loss is its definition written as nested loops.  Per sequence s of T steps, with
 * P_t the trainable router's distribution, P_t^ref the frozen snapshot router's, and E_{t-1} the
 * previous step's routed set (a constant for the purposes of the value):
 *
 *   m_t      = (1/K) sum_{k in E_{t-1}} P_t[k]                              (Eq. 2, reuse mass)
 *   rho      = (1/(T-1)) sum_{t=2..T} m_t ,  L_Reuse = -log(rho + 1e-8)     (Eq. 7)
 *   L_Trust  = (1/T) sum_t KL(P_t || P_t^ref)                               (Eq. 4, 5)
 *   SymKL(P,Q) = (KL(P||Q) + KL(Q||P)) / 2                                  (Eq. 8)
 *   L_Smooth = (1/(T-1)) sum_{t=2..T} SymKL(P_t, P_{t-1})                   (Eq. 9)
 *   L_Lag    = (1/(T-1)) sum_{t=2..T} (1/|D|) sum_{d in D, t-d >= 1} SymKL(P_t, P_{t-d})   (Eq. 10)
 *   Pbar_b   = mean of the W distributions of window b, b = 1..n, n = floor(T / W)          (Eq. 11)
 *   L_WS     = (1/n) sum_b H(Pbar_b),  H(P) = -sum_k P[k] log P[k]          (Eq. 12)
 *
 * Conventions where the formulas leave a case open: 0 log 0 = 0; T < 2 gives rho = 0 and
 * L_Smooth = L_Lag = 0; n = 0 gives L_WS = 0; the sums over t of Eq. 9-10 use 1-based steps, i.e.
 * every t whose partner t - d exists.  The weighted sum L_Loc (Eq. 6) and the warm-up factor are
 * the caller's arithmetic.
 *
 * Parity status: pinned by the CPU tests (closed forms for constant, uniform and identical
 * distributions, torch's kl_div and special.entr in fp64, the identity L_Lag = L_Smooth
 * for D = {1}).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

static double kl(const float *p, const float *q, int n)
{
    double s = 0.0;
    for (int k = 0; k < n; ++k)
        if (p[k] > 0.0f) s += (double)p[k] * (log((double)p[k]) - log((double)q[k]));
    return s;
}

static double symkl(const float *p, const float *q, int n) { return 0.5 * (kl(p, q, n) + kl(q, p, n)); }

/* out [S, 6]: rho, L_Reuse, L_Trust, L_Smooth, L_Lag, L_WS */
int oracle_remoe_losses(const float *probs, const float *probs_ref, const int32_t *idx, int64_t n_seq,
                        int64_t n_steps, int n_experts, int top_k, const int32_t *lags, int n_lags, int window,
                        double *out)
{
    if (!probs || !probs_ref || !idx || !out || n_experts < 1 || top_k < 1 || n_lags < 0 || window < 1) return -1;
    for (int i = 0; i < n_lags; ++i) if (lags[i] < 1) return -1;
    const int N = n_experts;
    const int64_t T = n_steps;
    for (int64_t s = 0; s < n_seq; ++s) {
        const float *P = probs + s * T * N, *Q = probs_ref + s * T * N;
        const int32_t *E = idx + s * T * top_k;
        double rho = 0.0, trust = 0.0, smooth = 0.0, lag = 0.0, ws = 0.0;
        for (int64_t t = 0; t < T; ++t) trust += kl(P + t * N, Q + t * N, N);
        if (T > 0) trust /= (double)T;
        for (int64_t t = 1; t < T; ++t) {
            double m = 0.0;
            for (int j = 0; j < top_k; ++j) m += (double)P[t * N + E[(t - 1) * top_k + j]];
            rho += m / (double)top_k;
            smooth += symkl(P + t * N, P + (t - 1) * N, N);
            double l = 0.0;
            for (int i = 0; i < n_lags; ++i)
                if (t - lags[i] >= 0) l += symkl(P + t * N, P + (t - lags[i]) * N, N);
            if (n_lags > 0) lag += l / (double)n_lags;
        }
        if (T > 1) { rho /= (double)(T - 1); smooth /= (double)(T - 1); lag /= (double)(T - 1); }
        const int64_t n = T / window;
        double *bar = (double *)malloc(sizeof(double) * (size_t)N);
        for (int64_t b = 0; b < n; ++b) {
            for (int k = 0; k < N; ++k) {
                double a = 0.0;
                for (int j = 0; j < window; ++j) a += (double)P[(b * window + j) * N + k];
                bar[k] = a / (double)window;
            }
            double h = 0.0;
            for (int k = 0; k < N; ++k) if (bar[k] > 0.0) h -= bar[k] * log(bar[k]);
            ws += h;
        }
        free(bar);
        if (n > 0) ws /= (double)n;
        double *o = out + s * 6;
        o[0] = rho; o[1] = -log(rho + 1e-8); o[2] = trust; o[3] = smooth; o[4] = lag; o[5] = ws;
    }
    return 0;
}
