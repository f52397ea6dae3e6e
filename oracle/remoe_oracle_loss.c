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
 * for D = {1}).  The gradient functions further down are pinned by reverse-mode differentiation
 * (torch.autograd, fp64) of the loss definitions written with tensor operations, by central
 * differences of oracle_remoe_losses itself, by the zero row sums a softmax gradient has, and the
 * gate gradient by torch's matmul.
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

/*
 * Gradient of a weighted sum of the regularisers with respect to the router logits, and the gate
 * gradient it induces.
 *
 * Per sequence, L = c[0] L_Reuse + c[1] L_Trust + c[2] L_Smooth + c[3] L_Lag + c[4] L_WS (the sum of
 * Eq. 3 / Eq. 6 with the caller's weights), P_t = softmax(z_t).  The partial derivatives of the
 * definitions above with respect to one entry P_t[k], every other entry held fixed:
 *
 *   L_Reuse :  -1 / ((rho + 1e-8) (T-1) K)   if t >= 2 and k in E_{t-1}, else 0   (E_{t-1} is a constant:
 *              the previous routed set is a stop-gradient target, Eq. 2)
 *   L_Trust :  (log P_t[k] - log P_t^ref[k] + 1) / T                              (P^ref is frozen, Eq. 4)
 *   SymKL(P, R) with respect to P[k]:  phi(P, R)[k] = (log P[k] - log R[k] + 1 - R[k] / P[k]) / 2,
 *              and, SymKL being symmetric, the same expression with the roles exchanged for R
 *   L_Smooth:  (phi(P_t, P_{t-1}) [t >= 2] + phi(P_t, P_{t+1}) [t < T]) / (T-1)   (no stop-gradient, Sec. 4.4)
 *   L_Lag   :  sum_{d in D} (phi(P_t, P_{t-d}) [t-d >= 1] + phi(P_t, P_{t+d}) [t+d <= T]) / ((T-1) |D|)
 *              (the paper does not mention a stop-gradient for Eq. 10; both arguments carry gradient,
 *              as in Eq. 9)
 *   L_WS    :  -(log Pbar_b[k] + 1) / (n W)   for t in a complete window b, else 0
 *
 * and through the softmax  dL/dz_t[k] = P_t[k] (g[k] - sum_j P_t[j] g[j]),  g = dL/dP_t.
 * Entries with P_t[k] = 0 get gradient 0 (the limit of P (log P + const)).  out [S, T, N] double.
 */
static double phi(double p, double r) { return 0.5 * (log(p) - log(r) + 1.0 - r / p); }

int oracle_remoe_loss_grad(const float *probs, const float *probs_ref, const int32_t *idx, int64_t n_seq,
                           int64_t n_steps, int n_experts, int top_k, const int32_t *lags, int n_lags, int window,
                           const double *coef, double *out)
{
    if (!probs || !probs_ref || !idx || !out || !coef || n_experts < 1 || top_k < 1 || n_lags < 0 || window < 1) return -1;
    for (int i = 0; i < n_lags; ++i) if (lags[i] < 1) return -1;
    const int N = n_experts;
    const int64_t T = n_steps;
    double *g = (double *)malloc(sizeof(double) * (size_t)N);
    double *bar = (double *)malloc(sizeof(double) * (size_t)N);
    for (int64_t s = 0; s < n_seq; ++s) {
        const float *P = probs + s * T * N, *Q = probs_ref + s * T * N;
        const int32_t *E = idx + s * T * top_k;
        double rho = 0.0;
        for (int64_t t = 1; t < T; ++t)
            for (int j = 0; j < top_k; ++j) rho += (double)P[t * N + E[(t - 1) * top_k + j]] / (double)top_k;
        if (T > 1) rho /= (double)(T - 1);
        const int64_t n = T / window;
        for (int64_t t = 0; t < T; ++t) {
            const float *p = P + t * N;
            for (int k = 0; k < N; ++k) g[k] = 0.0;
            if (t >= 1)
                for (int j = 0; j < top_k; ++j)   /* over the K entries of E_{t-1}, exactly as m_t sums them */
                    g[E[(t - 1) * top_k + j]] += coef[0] * -1.0 / ((rho + 1e-8) * (double)(T - 1) * (double)top_k);
            const int64_t b = t / window;
            if (b < n)
                for (int k = 0; k < N; ++k) {
                    double a = 0.0;
                    for (int j = 0; j < window; ++j) a += (double)P[(b * window + j) * N + k];
                    bar[k] = a / (double)window;
                }
            for (int k = 0; k < N; ++k) {
                const double pk = (double)p[k];
                if (!(pk > 0.0)) continue;
                g[k] += coef[1] * (log(pk) - log((double)Q[t * N + k]) + 1.0) / (double)T;
                if (T > 1) {
                    double sm = 0.0, lg = 0.0;
                    if (t >= 1) sm += phi(pk, (double)P[(t - 1) * N + k]);
                    if (t + 1 < T) sm += phi(pk, (double)P[(t + 1) * N + k]);
                    for (int i = 0; i < n_lags; ++i) {
                        if (t - lags[i] >= 0) lg += phi(pk, (double)P[(t - lags[i]) * N + k]);
                        if (t + lags[i] < T) lg += phi(pk, (double)P[(t + lags[i]) * N + k]);
                    }
                    g[k] += coef[2] * sm / (double)(T - 1);
                    if (n_lags > 0) g[k] += coef[3] * lg / ((double)(T - 1) * (double)n_lags);
                }
                if (b < n) g[k] += coef[4] * -(log(bar[k]) + 1.0) / ((double)n * (double)window);
            }
            double dot = 0.0;
            for (int k = 0; k < N; ++k) dot += (double)p[k] * g[k];
            for (int k = 0; k < N; ++k) out[(s * T + t) * N + k] = (double)p[k] * (g[k] - dot);
        }
    }
    free(g);
    free(bar);
    return 0;
}

/*
 * Gate gradient: z_t = W_r x_t, so dL/dW_r[e, h] = sum over all tokens of dz[t, e] x[t, h]
 * (the router has no bias, Sec. 3.1).  dz fp32 [T, N] (what the device path hands to its GEMM), x
 * fp32 [T, H] (bf16 inputs upcast exactly by the caller), out double [N, H].  With n_pick > 0 only the
 * entries pick[2 i] = e, pick[2 i + 1] = h are evaluated, into out[i].
 */
int oracle_gate_grad(const float *dz, const float *x, int64_t n_tokens, int n_experts, int hidden,
                     const int32_t *pick, int64_t n_pick, double *out)
{
    if (!dz || !x || !out || n_experts < 1 || hidden < 1) return -1;
    if (n_pick > 0) {
        for (int64_t i = 0; i < n_pick; ++i) {
            const int e = pick[2 * i], h = pick[2 * i + 1];
            if (e < 0 || e >= n_experts || h < 0 || h >= hidden) return -1;
            double a = 0.0;
            for (int64_t t = 0; t < n_tokens; ++t) a += (double)dz[t * n_experts + e] * (double)x[t * hidden + h];
            out[i] = a;
        }
        return 0;
    }
    for (int e = 0; e < n_experts; ++e)
        for (int h = 0; h < hidden; ++h) {
            double a = 0.0;
            for (int64_t t = 0; t < n_tokens; ++t) a += (double)dz[t * n_experts + e] * (double)x[t * hidden + h];
            out[(int64_t)e * hidden + h] = a;
        }
    return 0;
}
