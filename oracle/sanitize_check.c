/*
 * Driver for the sanitizer build of the CPU oracle (TEST INFRASTRUCTURE ONLY).
 *
 * oracle/build.py links this file with the oracle's sources under -fsanitize=address,undefined and a
 * CPU test runs the result: every oracle function is called on small seeded inputs, including the
 * shapes where index arithmetic is most likely to slip (one token, one expert, K = N_r, C < K,
 * repeated ids, a histogram shorter than the sums, lags longer than the sequence, empty traces).
 * Buffers are heap blocks of exactly the documented size, so a read or write one element past an
 * end is reported.  Exit status 0 means every call returned its expected status and the sanitizers
 * stayed silent.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_route(const void *, int, int64_t, int, const float *, int, int, int, int32_t *, double *, double *, double *, double *);
int oracle_experts_sparse(const void *, int, int, int, int, int, const int32_t *, const double *, const void *, const void *,
                          const void *, int, const void *, const void *, const void *, const float *, const int64_t *, int64_t,
                          double *);
int oracle_experts_dense_masked(const void *, int, int64_t, int, int, int, int, const int32_t *, const double *, const void *,
                                const void *, const void *, int, const void *, const void *, const void *, const float *, double *);
int oracle_trace_reuse(const int32_t *, int64_t, int64_t, int, int, uint8_t *, uint64_t *);
int oracle_lru_list(const int32_t *, int64_t, int64_t, int, int, int, uint64_t, uint8_t *, uint64_t *, uint64_t *);
int oracle_cache_policy(const int32_t *, int64_t, int64_t, int, int, int, int, uint64_t, uint8_t *, uint8_t *, uint8_t *,
                        uint64_t *, uint64_t *, uint64_t *);
int oracle_step_summary(const uint8_t *, int64_t, int64_t, int64_t, uint16_t *, uint64_t *, int64_t, int32_t *);
int oracle_balance(const int32_t *, int64_t, int64_t, int, int, uint32_t *, int32_t *, double *, double *);
int oracle_reroute_lru(const float *, int64_t, int64_t, int, int, int, float, int, int32_t *, double *, uint8_t *, uint64_t *);
int oracle_remoe_losses(const float *, const float *, const int32_t *, int64_t, int64_t, int, int, const int32_t *, int, int,
                        double *);
int oracle_remoe_loss_grad(const float *, const float *, const int32_t *, int64_t, int64_t, int, int, const int32_t *, int,
                           int, const double *, double *);
int oracle_gate_grad(const float *, const float *, int64_t, int, int, const int32_t *, int64_t, double *);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void)
{
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(rng_state >> 33);
}
static float rndf(void) { return ((float)(rnd() & 0xFFFF) / 65536.0f - 0.5f) * 0.2f; }

static void *blk(size_t n) { void *p = malloc(n ? n : 1); if (!p) exit(3); memset(p, 0, n); return p; }
static float *frand(size_t n) { float *p = blk(n * 4); for (size_t i = 0; i < n; ++i) p[i] = rndf(); return p; }
static uint16_t *brand(size_t n)
{
    uint16_t *p = blk(n * 2);
    for (size_t i = 0; i < n; ++i) { float f = rndf(); uint32_t u; memcpy(&u, &f, 4); p[i] = (uint16_t)(u >> 16); }
    return p;
}

static int fails = 0;
#define EXPECT(call, want)                                                                  \
    do {                                                                                    \
        int rc_ = (call);                                                                   \
        if (rc_ != (want)) { fprintf(stderr, "%s:%d: %s returned %d, expected %d\n", __FILE__, __LINE__, #call, rc_, (want)); ++fails; } \
    } while (0)

/* K distinct ids per step (or repeated ids when distinct == 0) */
static int32_t *trace(int64_t S, int64_t T, int K, int N, int distinct)
{
    int32_t *t = blk((size_t)(S * T * K) * 4);
    for (int64_t i = 0; i < S * T; ++i)
        for (int j = 0; j < K; ++j) {
            int e, again;
            do {
                e = (int)(rnd() % (uint32_t)N);
                again = 0;
                for (int q = 0; q < j && distinct; ++q) again |= (t[i * K + q] == e);
            } while (again);
            t[i * K + j] = e;
        }
    return t;
}

static void layer_case(int dtype, int64_t T, int H, int N, int I, int K, int renorm, int Is, int gate)
{
    const size_t es = dtype ? 2 : 4;
    void *x = dtype ? (void *)brand((size_t)T * H) : (void *)frand((size_t)T * H);
    float *wr = frand((size_t)N * H);
    void *wg = dtype ? (void *)brand((size_t)N * I * H) : (void *)frand((size_t)N * I * H);
    void *wu = dtype ? (void *)brand((size_t)N * I * H) : (void *)frand((size_t)N * I * H);
    void *wd = dtype ? (void *)brand((size_t)N * H * I) : (void *)frand((size_t)N * H * I);
    void *sg = Is ? (dtype ? (void *)brand((size_t)Is * H) : (void *)frand((size_t)Is * H)) : NULL;
    void *su = Is ? (dtype ? (void *)brand((size_t)Is * H) : (void *)frand((size_t)Is * H)) : NULL;
    void *sd = Is ? (dtype ? (void *)brand((size_t)H * Is) : (void *)frand((size_t)H * Is)) : NULL;
    float *sc = (Is && gate) ? frand((size_t)H) : NULL;
    int32_t *idx = blk((size_t)T * K * 4);
    double *w = blk((size_t)T * K * 8), *margin = blk((size_t)T * 8);
    double *probs = blk((size_t)T * N * 8), *logits = blk((size_t)T * N * 8);
    (void)es;
    EXPECT(oracle_route(x, dtype, T, H, wr, N, K, renorm, idx, w, margin, probs, logits), 0);
    EXPECT(oracle_route(x, dtype, T, H, wr, N, K, renorm, idx, w, NULL, NULL, NULL), 0);
    double *y = blk((size_t)T * H * 8), *yd = blk((size_t)T * H * 8);
    EXPECT(oracle_experts_sparse(x, dtype, H, N, I, K, idx, w, wg, wu, wd, Is, sg, su, sd, sc, NULL, T, y), 0);
    EXPECT(oracle_experts_dense_masked(x, dtype, T, H, N, I, K, idx, w, wg, wu, wd, Is, sg, su, sd, sc, yd), 0);
    for (int64_t i = 0; i < T * H; ++i)
        if (fabs(y[i] - yd[i]) > 1e-12 * (1.0 + fabs(y[i]))) { fprintf(stderr, "sparse != dense at %lld\n", (long long)i); ++fails; break; }
    if (T > 1) {   /* a selection of tokens (rows of x, idx and w alike): the last and the first */
        int64_t sel[2] = {T - 1, 0};
        double *ys = blk((size_t)2 * H * 8);
        EXPECT(oracle_experts_sparse(x, dtype, H, N, I, K, idx, w, wg, wu, wd, Is, sg, su, sd, sc, sel, 2, ys), 0);
        for (int h = 0; h < H; ++h)
            if (ys[h] != y[(T - 1) * H + h] || ys[H + h] != y[h]) { fprintf(stderr, "selected rows differ\n"); ++fails; break; }
        free(ys);
    }
    free(x); free(wr); free(wg); free(wu); free(wd); free(sg); free(su); free(sd); free(sc);
    free(idx); free(w); free(margin); free(probs); free(logits); free(y); free(yd);
}

static void trace_case(int64_t S, int64_t T, int K, int N, int C, int distinct)
{
    int32_t *tr = trace(S, T, K, N, distinct);
    uint8_t *ov = blk((size_t)(S * T)), *miss = blk((size_t)(S * T)), *uq = blk((size_t)(S * T)), *ht = blk((size_t)(S * T));
    uint64_t *sum = blk((size_t)S * 8), *tot = blk((size_t)S * 8), *tu = blk((size_t)S * 8), *by = blk((size_t)S * 8);
    EXPECT(oracle_trace_reuse(tr, S, T, K, N, ov, sum), 0);
    EXPECT(oracle_lru_list(tr, S, T, K, N, C, 9437184ull, miss, tot, by), 0);
    for (int p = 0; p < 4; ++p) EXPECT(oracle_cache_policy(tr, S, T, K, N, C, p, 7ull, miss, uq, ht, tot, tu, by), 0);
    uint32_t *load = blk((size_t)S * N * 4);
    int32_t *used = blk((size_t)S * 4);
    double *ent = blk((size_t)S * 8), *cv = blk((size_t)S * 8);
    EXPECT(oracle_balance(tr, S, T, K, N, load, used, ent, cv), 0);
    /* the miss table of the S traces read as S "layers" of one sequence: per-step sums, short histogram */
    uint16_t *all = blk((size_t)T * 2);
    for (int64_t hl = 1; hl <= 3; ++hl) {
        uint64_t *hist = blk((size_t)hl * 8);
        int32_t pct[3];
        EXPECT(oracle_step_summary(miss, S, 1, T, all, hist, hl, pct), 0);
        free(hist);
    }
    if (T > 0 && S > 0) {
        tr[0] = N;   /* an id out of range is refused, not used as an index */
        EXPECT(oracle_trace_reuse(tr, S, T, K, N, ov, sum), -1);
        EXPECT(oracle_lru_list(tr, S, T, K, N, C, 1ull, miss, tot, by), -1);
        EXPECT(oracle_cache_policy(tr, S, T, K, N, C, 1, 1ull, miss, uq, ht, tot, tu, by), -1);
        EXPECT(oracle_balance(tr, S, T, K, N, load, used, ent, cv), -1);
    }
    free(tr); free(ov); free(miss); free(uq); free(ht); free(sum); free(tot); free(tu); free(by);
    free(load); free(used); free(ent); free(cv); free(all);
}

static float *softmax_rows(int64_t rows, int N)
{
    float *p = blk((size_t)rows * N * 4);
    for (int64_t r = 0; r < rows; ++r) {
        double s = 0.0;
        for (int e = 0; e < N; ++e) { p[r * N + e] = expf(20.0f * rndf()); s += p[r * N + e]; }
        for (int e = 0; e < N; ++e) p[r * N + e] = (float)(p[r * N + e] / s);
    }
    return p;
}

static void loss_case(int64_t S, int64_t T, int N, int K, int window)
{
    float *p = softmax_rows(S * T, N), *pr = softmax_rows(S * T, N);
    int32_t *idx = trace(S, T, K, N, 1);
    const int32_t lags[5] = {1, 2, 4, 8, 16};
    const double coef[5] = {1.0, 0.5, 0.25, 0.125, 2.0};
    double *out = blk((size_t)S * 6 * 8), *dz = blk((size_t)(S * T * N) * 8);
    EXPECT(oracle_remoe_losses(p, pr, idx, S, T, N, K, lags, 5, window, out), 0);
    EXPECT(oracle_remoe_loss_grad(p, pr, idx, S, T, N, K, lags, 5, window, coef, dz), 0);
    EXPECT(oracle_remoe_losses(p, pr, idx, S, T, N, K, lags, 0, window, out), 0);
    /* rerouting on the same probabilities */
    int32_t *ri = blk((size_t)(S * T * K) * 4);
    double *rw = blk((size_t)(S * T * K) * 8);
    uint8_t *rm = blk((size_t)(S * T));
    uint64_t *rt = blk((size_t)S * 8);
    EXPECT(oracle_reroute_lru(p, S, T, N, K, K + 1, 3.0f, 1, ri, rw, rm, rt), 0);
    EXPECT(oracle_reroute_lru(p, S, T, N, K, 1, 1.0f, 0, ri, rw, rm, rt), 0);
    /* gate gradient: every entry, then two picked entries */
    const int H = 24;
    float *dzf = frand((size_t)(S * T) * N), *x = frand((size_t)(S * T) * H);
    double *dw = blk((size_t)N * H * 8), *dw2 = blk(2 * 8);
    EXPECT(oracle_gate_grad(dzf, x, S * T, N, H, NULL, 0, dw), 0);
    const int32_t pick[4] = {0, 0, N - 1, H - 1};
    EXPECT(oracle_gate_grad(dzf, x, S * T, N, H, pick, 2, dw2), 0);
    free(p); free(pr); free(idx); free(out); free(dz); free(ri); free(rw); free(rm); free(rt);
    free(dzf); free(x); free(dw); free(dw2);
}

int main(void)
{
    layer_case(0, 7, 48, 5, 20, 2, 0, 0, 0);        /* fp32, odd sizes */
    layer_case(0, 1, 32, 1, 8, 1, 1, 0, 0);         /* one token, one expert */
    layer_case(1, 9, 64, 6, 24, 6, 1, 0, 0);        /* bf16, K = N_r */
    layer_case(1, 5, 64, 8, 16, 3, 0, 40, 1);       /* gated shared expert */
    layer_case(0, 4, 32, 4, 8, 2, 0, 16, 0);        /* ungated shared expert */
    trace_case(3, 40, 2, 9, 4, 1);
    trace_case(2, 25, 6, 20, 3, 1);                 /* C < K */
    trace_case(2, 30, 4, 12, 5, 0);                 /* repeated ids */
    trace_case(1, 1, 3, 8, 2, 1);                   /* a single step */
    trace_case(2, 17, 5, 5, 9, 1);                  /* K = N_r, C > N_r */
    trace_case(1, 0, 2, 4, 2, 1);                   /* an empty trace */
    loss_case(2, 12, 8, 2, 4);
    loss_case(1, 1, 4, 1, 3);                       /* one step: no partner, no full window */
    loss_case(1, 40, 16, 4, 7);                     /* lags up to 16, ragged last window */
    if (fails) { fprintf(stderr, "sanitize_check: %d unexpected result(s)\n", fails); return 1; }
    printf("sanitize_check ok\n");
    return 0;
}
