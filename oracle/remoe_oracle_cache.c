/*
 * CPU oracle, second file: the rest of the paper's expert-cache simulator and the routing-balance
 * statistics.
 *
 * TEST INFRASTRUCTURE ONLY (see remoe_oracle.c).  Plain loops over sets held as arrays, one cold
 * cache per trace, no code shared with the HIP library.
 *
 * What follows which passage of the paper:
 *   - per-step token / unique hits and misses against the resident set BEFORE the step, totals,
 *     uHR = sum H_uniq / sum T_uniq (App. E.2, "Per-step hits and misses", "Aggregate metrics");
 *   - the update rule "depends on the chosen policy (LRU/LFU/FIFO)" (App. E.2, "Cache state") and
 *     Belady's MIN is evaluated "under the same reset protocol" (App. F.1).  The paper gives no
 *     rule beyond the policies' names; the readings taken are stated at oracle_cache_policy;
 *   - per-step sums over all MoE layers and their P50/P95/P99 (App. E.2, "Per-step (edge)
 *     reporting");
 *   - expert-load balance of a trace: normalised routing entropy, coefficient of variation of the
 *     expert loads, distinct experts used (Sec. 5.2 names these quantities without defining them;
 *     the definitions taken are stated at oracle_balance).
 *
 * Parity status: pinned by the CPU tests (textbook single-request FIFO / LFU simulations, the list
 * LRU of the first file, exhaustive search for the minimum number of misses on tiny traces, the
 * accounting identity of the paper's full cache table, numpy's inverted-CDF percentile, closed forms
 * of entropy and variation for uniform and one-hot loads).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { POLICY_LRU = 0, POLICY_FIFO = 1, POLICY_LFU = 2, POLICY_BELADY = 3 };

/* Is candidate a kept in preference to candidate b?  (Both are in the cache or were just requested.) */
static int keep_before(int policy, int a, int b, const int64_t *last, const int64_t *ins,
                       const int64_t *freq, const int64_t *next_use)
{
    switch (policy) {
    case POLICY_LRU:      /* more recently used first; inside one step the higher id counts as later */
        if (last[a] != last[b]) return last[a] > last[b];
        return a > b;
    case POLICY_FIFO:     /* more recently brought in first; inside one step the higher id counts as later */
        if (ins[a] != ins[b]) return ins[a] > ins[b];
        return a > b;
    case POLICY_LFU:      /* more often requested first; then more recently used; then the higher id */
        if (freq[a] != freq[b]) return freq[a] > freq[b];
        if (last[a] != last[b]) return last[a] > last[b];
        return a > b;
    default:              /* Belady: needed again sooner first; among equals the lower id */
        if (next_use[a] != next_use[b]) return next_use[a] < next_use[b];
        return a < b;
    }
}

/*
 * One cache of `capacity` experts per trace, cold at the start of the trace (App. E.2).  A step:
 *   U = distinct requested ids; token hits = requested slots whose expert is resident (with
 *   multiplicity); unique misses = |U \ resident| -- all against the state before the step;
 *   then every expert of U is in the cache (a missing one has just been fetched), the bookkeeping
 *   of the policy is updated, and while more than `capacity` experts are held one is dropped:
 *   the one keep_before ranks last among the held experts that this step did NOT request.  An
 *   expert served in a step is not evicted before the step is over, and "LRU/LFU/FIFO satisfy
 *   E_t in C_{t+1} under C >= K by evicting experts not in E_t" (App. A, step atomicity and
 *   admission; Prop. 3.1's bound miss_t <= K - |E_t n E_{t-1}| rests on it).  Only when every held
 *   expert was requested by this step (more distinct requests than capacity, outside the
 *   proposition) does the ranking run over the requested ones.
 * Readings (the paper names the policies only):
 *   LRU    as in oracle_lru_list (recency key (step, id));
 *   FIFO   age = step at which the expert was last brought in; a hit does not renew it;
 *   LFU    frequency = number of steps of the trace so far that requested the expert (kept across
 *          evictions), ties to the more recently used;
 *   Belady among the experts the step did not request, the one whose next request lies farthest
 *          ahead goes first (never again = farthest), ties to the higher id.
 */
int oracle_cache_policy(const int32_t *idx, int64_t n_seq, int64_t n_steps, int top_k, int n_experts,
                        int capacity, int policy, uint64_t expert_bytes,
                        uint8_t *out_miss, uint8_t *out_uniq, uint8_t *out_hit_tok,
                        uint64_t *out_total_miss, uint64_t *out_total_uniq, uint64_t *out_bytes)
{
    if (!idx || !out_miss || !out_uniq || !out_hit_tok || !out_total_miss || !out_total_uniq || !out_bytes) return -1;
    if (top_k < 1 || n_experts < 1 || capacity < 1 || policy < 0 || policy > 3) return -1;
    for (int64_t i = 0; i < n_seq * n_steps * top_k; ++i)
        if (idx[i] < 0 || idx[i] >= n_experts) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t s = 0; s < n_seq; ++s) {
        const int32_t *tr = idx + s * n_steps * top_k;
        uint8_t *resident = (uint8_t *)calloc((size_t)n_experts, 1);
        uint8_t *req = (uint8_t *)calloc((size_t)n_experts, 1);
        int64_t *last = (int64_t *)malloc(sizeof(int64_t) * (size_t)n_experts);
        int64_t *ins = (int64_t *)malloc(sizeof(int64_t) * (size_t)n_experts);
        int64_t *freq = (int64_t *)calloc((size_t)n_experts, sizeof(int64_t));
        int64_t *next_use = (int64_t *)malloc(sizeof(int64_t) * (size_t)n_experts);
        for (int e = 0; e < n_experts; ++e) { last[e] = -1; ins[e] = -1; next_use[e] = n_steps; }
        uint64_t total = 0, total_u = 0;
        for (int64_t t = 0; t < n_steps; ++t) {
            const int32_t *e = tr + t * top_k;
            memset(req, 0, (size_t)n_experts);
            int hit_tok = 0;
            for (int j = 0; j < top_k; ++j) { req[e[j]] = 1; hit_tok += resident[e[j]]; }
            int n_u = 0, miss = 0;
            for (int q = 0; q < n_experts; ++q) { n_u += req[q]; miss += req[q] && !resident[q]; }
            out_miss[s * n_steps + t] = (uint8_t)miss;
            out_uniq[s * n_steps + t] = (uint8_t)n_u;
            out_hit_tok[s * n_steps + t] = (uint8_t)hit_tok;
            total += (uint64_t)miss;
            total_u += (uint64_t)n_u;
            /* serve the step */
            for (int q = 0; q < n_experts; ++q) {
                if (!req[q]) continue;
                if (!resident[q]) ins[q] = t;
                resident[q] = 1;
                last[q] = t;
                freq[q] += 1;
            }
            if (policy == POLICY_BELADY) {
                /* next request of every held expert after step t: scan the future, as the definition says */
                for (int q = 0; q < n_experts; ++q) {
                    if (!resident[q]) continue;
                    int64_t nu = n_steps;
                    for (int64_t f = t + 1; f < n_steps && nu == n_steps; ++f)
                        for (int j = 0; j < top_k; ++j)
                            if (tr[f * top_k + j] == q) { nu = f; break; }
                    next_use[q] = nu;
                }
            }
            int held = 0;
            for (int q = 0; q < n_experts; ++q) held += resident[q];
            while (held > capacity) {
                int victim = -1;
                for (int pass = 0; pass < 2 && victim < 0; ++pass) {   /* pass 0: experts outside this step's request */
                    for (int q = 0; q < n_experts; ++q) {
                        if (!resident[q] || (pass == 0 && req[q])) continue;
                        if (victim < 0 || keep_before(policy, victim, q, last, ins, freq, next_use)) victim = q;
                    }
                }
                resident[victim] = 0;
                --held;
            }
        }
        out_total_miss[s] = total;
        out_total_uniq[s] = total_u;
        out_bytes[s] = total * expert_bytes;
        free(resident); free(req); free(last); free(ins); free(freq); free(next_use);
    }
    return 0;
}

/*
 * Per-step sums over the MoE layers of one run and their percentiles (App. E.2, "Per-step (edge)
 * reporting"): all[s, t] = sum over layers of miss[l, s, t]; hist[v] = number of steps with
 * all = v; percentile p (p50, p95, p99) by the inverted empirical distribution: the smallest
 * value v whose cumulative count reaches p percent of the steps (the paper does not say which
 * percentile estimator it uses; this one stays on observed integer values).
 */
int oracle_step_summary(const uint8_t *miss, int64_t n_layers, int64_t n_seq, int64_t n_steps,
                        uint16_t *out_all, uint64_t *out_hist, int64_t hist_len, int32_t *out_pct)
{
    if (!miss || !out_all || !out_hist || !out_pct || hist_len < 1) return -1;
    const int64_t n = n_seq * n_steps;
    for (int64_t v = 0; v < hist_len; ++v) out_hist[v] = 0;
    for (int64_t i = 0; i < n; ++i) {
        uint32_t a = 0;
        for (int64_t l = 0; l < n_layers; ++l) a += miss[l * n + i];
        if (a > 65535u) return -2;
        out_all[i] = (uint16_t)a;
        out_hist[(int64_t)a < hist_len ? (int64_t)a : hist_len - 1] += 1;   /* sums beyond the table share its last bin */
    }
    const int pcts[3] = {50, 95, 99};
    for (int k = 0; k < 3; ++k) {
        /* smallest v with 100 * cum(v) >= p * n */
        uint64_t cum = 0;
        int32_t ans = -1;
        for (int64_t v = 0; v < hist_len && ans < 0; ++v) {
            cum += out_hist[v];
            if (n > 0 && 100 * cum >= (uint64_t)pcts[k] * (uint64_t)n) ans = (int32_t)v;
        }
        out_pct[k] = ans;
    }
    return 0;
}

/*
 * Expert-load balance of each trace.  load[e] = number of routed slots (step, j) that name expert e;
 * with p_e = load[e] / sum(load):
 *   entropy = -sum_e p_e ln p_e / ln N_r        (0 ln 0 = 0; 1 = perfectly even, 0 = one expert; 0 when N_r = 1)
 *   cv      = sqrt( mean_e (load[e] - m)^2 ) / m,  m = mean_e load[e]     (population form; 0 = even)
 *   used    = number of experts with load > 0.
 * An empty trace gives entropy = cv = 0, used = 0.
 */
int oracle_balance(const int32_t *idx, int64_t n_seq, int64_t n_steps, int top_k, int n_experts,
                   uint32_t *out_load, int32_t *out_used, double *out_entropy, double *out_cv)
{
    if (!idx || !out_load || !out_used || !out_entropy || !out_cv) return -1;
    for (int64_t i = 0; i < n_seq * n_steps * top_k; ++i)
        if (idx[i] < 0 || idx[i] >= n_experts) return -1;
    for (int64_t s = 0; s < n_seq; ++s) {
        uint32_t *load = out_load + s * n_experts;
        for (int e = 0; e < n_experts; ++e) load[e] = 0;
        for (int64_t i = 0; i < n_steps * top_k; ++i) load[idx[s * n_steps * top_k + i]] += 1;
        const double total = (double)n_steps * (double)top_k;
        int used = 0;
        double h = 0.0, var = 0.0;
        const double m = total / (double)n_experts;
        for (int e = 0; e < n_experts; ++e) {
            if (load[e] > 0) {
                ++used;
                const double p = (double)load[e] / total;
                h -= p * log(p);
            }
            var += ((double)load[e] - m) * ((double)load[e] - m);
        }
        out_used[s] = used;
        out_entropy[s] = (total > 0 && n_experts > 1) ? h / log((double)n_experts) : 0.0;
        out_cv[s] = (total > 0) ? sqrt(var / (double)n_experts) / m : 0.0;
    }
    return 0;
}

/*
 * Cache-aware rerouting at inference time (App. G, "Setup"): a residency bonus beta is added to the
 * pre-Top-K router scores of the experts that are in the (LRU) cache, beta = 0 being the unmodified
 * router.  The routing of step t therefore depends on the cache left by steps < t, and the cache
 * on the routing: one sequential pass per trace, cold at its start.
 * Readings (the appendix gives the idea only):
 *   - the bonus is additive on the logits.  With P = softmax(logits) that is the same ordering as
 *     P_e * exp(beta) for resident experts against P_e for the others, which is the form used here
 *     (`factor` = exp(beta), applied in fp32 to fp32 probabilities: the selection is decided in
 *     that precision on both sides); ties go to the lower id;
 *   - the selected experts keep their unmodified probabilities as gate weights (the intervention
 *     moves the choice, not the mixture), divided by their sum when `renorm`;
 *   - the cache is the LRU of oracle_lru_list (misses against the state before the step, the
 *     step's experts touched in ascending id).
 * Outputs: idx [S,T,K] (descending boosted score), w [S,T,K] fp64, miss [S,T], total_miss [S].
 */
int oracle_reroute_lru(const float *probs, int64_t n_seq, int64_t n_steps, int n_experts, int top_k,
                       int capacity, float factor, int renorm,
                       int32_t *out_idx, double *out_w, uint8_t *out_miss, uint64_t *out_total_miss)
{
    if (!probs || !out_idx || !out_w || !out_miss || !out_total_miss) return -1;
    if (top_k < 1 || top_k > n_experts || capacity < 1) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t s = 0; s < n_seq; ++s) {
        int32_t *lst = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_experts + top_k));   /* resident ids, least recent first */
        float *score = (float *)malloc(sizeof(float) * (size_t)n_experts);
        uint8_t *taken = (uint8_t *)malloc((size_t)n_experts);
        int len = 0;
        uint64_t total = 0;
        for (int64_t t = 0; t < n_steps; ++t) {
            const float *p = probs + (s * n_steps + t) * n_experts;
            for (int e = 0; e < n_experts; ++e) {
                int resident = 0;
                for (int r = 0; r < len; ++r) resident |= (lst[r] == e);
                const volatile float boosted = p[e] * factor;      /* one fp32 multiply, rounded to fp32 */
                score[e] = resident ? boosted : p[e];
                taken[e] = 0;
            }
            int32_t *sel = out_idx + (s * n_steps + t) * top_k;
            double wsum = 0.0;
            for (int j = 0; j < top_k; ++j) {          /* K times: the largest remaining score, lowest id first */
                int best = -1;
                for (int e = 0; e < n_experts; ++e)
                    if (!taken[e] && (best < 0 || score[e] > score[best])) best = e;
                taken[best] = 1;
                sel[j] = best;
                wsum += (double)p[best];
            }
            for (int j = 0; j < top_k; ++j)
                out_w[(s * n_steps + t) * top_k + j] = renorm ? (double)p[sel[j]] / wsum : (double)p[sel[j]];
            /* LRU step on the selected set (distinct by construction) */
            int miss = 0;
            for (int e = 0; e < n_experts; ++e) {
                if (!taken[e]) continue;
                int found = 0;
                for (int r = 0; r < len; ++r) found |= (lst[r] == e);
                miss += !found;
            }
            for (int e = 0; e < n_experts; ++e) {      /* ascending id: move to the most-recent end */
                if (!taken[e]) continue;
                int r = 0;
                while (r < len && lst[r] != e) ++r;
                if (r < len) { for (; r + 1 < len; ++r) lst[r] = lst[r + 1]; --len; }
                lst[len++] = e;
            }
            if (len > capacity) {
                const int drop = len - capacity;
                for (int r = 0; r + drop < len; ++r) lst[r] = lst[r + drop];
                len = capacity;
            }
            out_miss[s * n_steps + t] = (uint8_t)miss;
            total += (uint64_t)miss;
        }
        out_total_miss[s] = total;
        free(lst); free(score); free(taken);
    }
    return 0;
}
