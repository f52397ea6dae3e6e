// The rest of the paper's expert-cache simulator on routing traces, and routing-balance statistics.
//
// cache_policy_kernel: per-layer expert cache of capacity C under LRU, FIFO, LFU or Belady's MIN
// (App. E.2 "Cache state": the update rule depends on the policy, the hit / miss definitions do
// not; App. F.1 evaluates Belady under the same per-request resets).  Per step it reports the
// unique misses |U_t \ C_t| and the token hits against the resident set BEFORE the step, and |U_t|
// (App. E.2, "Per-step hits and misses"); per trace the totals that give #uMiss and uHR.
// These policies carry state from step to step (unlike LRU, whose resident set is a function of
// the last requests alone), so a trace is walked in order: one wavefront per trace, the resident set
// a 128-bit mask in wave-uniform registers, lane l holding the retention keys of experts l and
// l + 64.  After a step every requested expert is held; while more than C are held, the one with the
// smallest key among those the step did not request is dropped (a wavefront-wide minimum of the
// secondary key, which ends in the expert id and therefore names the victim; LFU takes the minimum
// of its primary key first).  Keys (larger = kept longer):
//   LRU    (step of last use, id)                 FIFO  (step of last fetch, id)
//   LFU    requests so far, then (step of last use, id)
//   Belady (steps_total - step of next request, 127 - id): the next request farthest ahead goes first
// The next-request table of Belady comes from next_use_kernel, a backward walk over the same trace.
//
// step_summary_kernel / step_percentile_kernel: per-step sums of a miss table over the MoE layers,
// their histogram and P50 / P95 / P99 (App. E.2, "Per-step (edge) reporting").
//
// reroute_kernel: cache-aware rerouting at inference time (App. G): experts resident in the LRU cache
// get a bonus on their pre-top-k score, so each step's routing depends on the cache the earlier
// steps left.  Same walk as above, one wavefront per trace; the top-k of a step is K rounds of
// wavefront maximum over the boosted scores.
//
// balance_kernel: expert loads of a trace, experts used, normalised routing entropy and the
// coefficient of variation of the loads (the quantities Sec. 5.2 tracks to show that routing stays
// balanced).
#include "common.h"
#include "topk.h"

namespace remoe {

namespace {

constexpr int CP_BATCH = 64;            // steps staged in LDS at a time
constexpr int CP_MAX_K = 64;
constexpr uint32_t CP_NONE = 0xFFFFFFFFu;

// rows [t0, t0 + n) of a [T, K] int32 table -> LDS, coalesced
__device__ __forceinline__ void stage_rows(const int32_t *__restrict__ table, int64_t t0, int n, int K, int32_t *lds)
{
    const int lane = threadIdx.x & 63;
    for (int q = lane; q < n * K; q += 64) lds[q] = table[t0 * K + q];
}

// Belady: nxt[t, j] = first step after t that requests expert idx[t, j] again, or T (never).
// A backward walk, one wavefront per trace: seen[e] (LDS) is the earliest request of expert e among
// the steps already walked; lane j looks slot j's expert up and then enters the step itself.  One
// wavefront's LDS accesses are served in program order, so the look-ups of a step see the table as
// the later steps left it; a repeated id reads and writes the same values twice.
__global__ __launch_bounds__(64) void next_use_kernel(const int32_t *__restrict__ idx, int64_t T, int K, int N,
                                                      int32_t *__restrict__ nxt)
{
    __shared__ int32_t ids[CP_BATCH * CP_MAX_K];
    __shared__ int32_t outs[CP_BATCH * CP_MAX_K];
    __shared__ int32_t seen[128];
    const int64_t s = blockIdx.x;
    const int lane = threadIdx.x;
    const int32_t *tr = idx + s * T * K;
    int32_t *no = nxt + s * T * K;
    seen[lane] = (int32_t)T;
    seen[lane + 64] = (int32_t)T;
    for (int64_t hi = T; hi > 0; hi -= CP_BATCH) {
        const int64_t t0 = hi >= CP_BATCH ? hi - CP_BATCH : 0;
        const int n = (int)(hi - t0);
        stage_rows(tr, t0, n, K, ids);
        __syncthreads();
        for (int tt = n - 1; tt >= 0; --tt) {
            if (lane < K) {
                const int e = ids[tt * K + lane];
                const bool valid = e >= 0 && e < N;
                outs[tt * K + lane] = valid ? seen[e] : (int32_t)T;
                if (valid) seen[e] = (int32_t)(t0 + tt);
            }
        }
        __syncthreads();
        for (int q = lane; q < n * K; q += 64) no[t0 * K + q] = outs[q];
        __syncthreads();
    }
}

// lane `l` of a per-lane register (l wave-uniform)
__device__ __forceinline__ uint32_t get_lane(uint32_t reg, int l)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return (uint32_t)__builtin_amdgcn_readlane((int)reg, l);
#else
    (void)l;
    return reg;
#endif
}
__device__ __forceinline__ bool bit_of(unsigned long long lo, unsigned long long hi, int e)
{
    return (((e < 64 ? lo : hi) >> (e & 63)) & 1ull) != 0ull;
}

// The walk is sequential per trace and one wavefront has nothing to hide a dependent instruction's
// latency behind, so the step is kept short: the sets (resident, requested, evictable) are 128-bit
// masks in wave-uniform registers and all set arithmetic is scalar; only the retention keys are
// per lane.  A batch of 64 steps is staged in LDS and lane l first builds the request mask of step
// l (one pass, all steps at once); the walk then fetches a step's mask with four lane reads.  A key
// ends in the expert id, so the wavefront minimum names its victim without a search.
template <int POLICY>
__global__ __launch_bounds__(64) void cache_policy_kernel(const int32_t *__restrict__ idx, int64_t T, int K, int N, int C,
                                                          unsigned long long expert_bytes,
                                                          const int32_t *__restrict__ nxt,
                                                          uint8_t *__restrict__ out_miss, uint8_t *__restrict__ out_uniq,
                                                          uint8_t *__restrict__ out_hit_tok,
                                                          unsigned long long *__restrict__ out_total_miss,
                                                          unsigned long long *__restrict__ out_total_uniq,
                                                          unsigned long long *__restrict__ out_bytes)
{
    __shared__ int32_t ids[CP_BATCH * CP_MAX_K];
    __shared__ int32_t nus[(POLICY == REMOE_CACHE_BELADY) ? CP_BATCH * CP_MAX_K : 1];
    __shared__ uint32_t kb[(POLICY == REMOE_CACHE_BELADY) ? 128 : 1];
    const int64_t s = blockIdx.x;
    const int lane = threadIdx.x;
    const int32_t *tr = idx + s * T * K;
    unsigned long long res_lo = 0ull, res_hi = 0ull;          // resident experts 0..63, 64..127 (wave-uniform)
    uint32_t khi0 = 0, khi1 = 0, klo0 = 0, klo1 = 0;          // keys of experts lane, lane + 64
    unsigned long long total = 0, total_u = 0;
    for (int64_t t0 = 0; t0 < T; t0 += CP_BATCH) {
        const int n = (int)((T - t0 < CP_BATCH) ? T - t0 : CP_BATCH);
        stage_rows(tr, t0, n, K, ids);
        if (POLICY == REMOE_CACHE_BELADY) stage_rows(nxt + s * T * K, t0, n, K, nus);
        __syncthreads();
        // request mask of step t0 + lane
        unsigned long long m_lo = 0ull, m_hi = 0ull;
        if (lane < n) {
            for (int j = 0; j < K; ++j) {
                const int e = ids[lane * K + j];
                if (e >= 0 && e < N) {
                    if (e < 64) m_lo |= 1ull << e;
                    else m_hi |= 1ull << (e - 64);
                }
            }
        }
        const uint32_t m0 = (uint32_t)m_lo, m1 = (uint32_t)(m_lo >> 32), m2 = (uint32_t)m_hi, m3 = (uint32_t)(m_hi >> 32);
        uint32_t o_miss = 0, o_uniq = 0, o_hit = 0;           // results of step t0 + lane
        for (int tt = 0; tt < n; ++tt) {
            const uint32_t t = (uint32_t)(t0 + tt);
            const unsigned long long req_lo = ((unsigned long long)get_lane(m1, tt) << 32) | get_lane(m0, tt);
            const unsigned long long req_hi = ((unsigned long long)get_lane(m3, tt) << 32) | get_lane(m2, tt);
            // token hits count a repeated id every time: lane j looks at slot j
            const int ej = lane < K ? ids[tt * K + lane] : -1;
            const int hit_tok = __popcll(__ballot(ej >= 0 && ej < N && bit_of(res_lo, res_hi, ej)));
            const int n_u = __popcll(req_lo) + __popcll(req_hi);
            const int miss = __popcll(req_lo & ~res_lo) + __popcll(req_hi & ~res_hi);
            // serve the step: every requested expert is held now; refresh its key
            const bool req0 = ((req_lo >> lane) & 1ull) != 0ull, req1 = ((req_hi >> lane) & 1ull) != 0ull;
            const uint32_t stamp = ((t + 1u) << 7);
            if (POLICY == REMOE_CACHE_LRU || POLICY == REMOE_CACHE_LFU) {
                if (req0) klo0 = stamp | (uint32_t)lane;
                if (req1) klo1 = stamp | (uint32_t)(lane + 64);
            }
            if (POLICY == REMOE_CACHE_FIFO) {
                const bool res0 = ((res_lo >> lane) & 1ull) != 0ull, res1 = ((res_hi >> lane) & 1ull) != 0ull;
                if (req0 && !res0) klo0 = stamp | (uint32_t)lane;
                if (req1 && !res1) klo1 = stamp | (uint32_t)(lane + 64);
            }
            if (POLICY == REMOE_CACHE_LFU) {
                khi0 += req0 ? 1u : 0u;
                khi1 += req1 ? 1u : 0u;
            }
            if (POLICY == REMOE_CACHE_BELADY) {
                // lane j posts the key of slot j's expert, the lanes that own a requested expert pick theirs
                // up (one wavefront: its LDS accesses are served in program order; a repeated id posts the
                // same key twice)
                if (ej >= 0 && ej < N) kb[ej] = (((uint32_t)T - (uint32_t)nus[tt * K + lane]) << 7) | (uint32_t)(127 - ej);
                if (req0) klo0 = kb[lane];
                if (req1) klo1 = kb[lane + 64];
            }
            res_lo |= req_lo;
            res_hi |= req_hi;
            int held = __popcll(res_lo) + __popcll(res_hi);
            // Victims come from the held experts this step did not request: an expert served in a step
            // stays until the step is over (App. A, step atomicity and admission: E_t is part of the
            // next resident set whenever C >= K).  Only a step with more distinct requests than C
            // leaves none of those, and then the ranking runs over the requested ones.
            unsigned long long free_lo = res_lo & ~req_lo, free_hi = res_hi & ~req_hi;
            while (held > C) {
                const bool any_free = (free_lo | free_hi) != 0ull;
                const unsigned long long c_lo = any_free ? free_lo : res_lo, c_hi = any_free ? free_hi : res_hi;
                bool c0 = ((c_lo >> lane) & 1ull) != 0ull, c1 = ((c_hi >> lane) & 1ull) != 0ull;
                if (POLICY == REMOE_CACHE_LFU) {
                    const uint32_t a0 = c0 ? khi0 : CP_NONE, a1 = c1 ? khi1 : CP_NONE;
                    const uint32_t mhi = wave_min_u32(a0 < a1 ? a0 : a1);
                    c0 = c0 && khi0 == mhi;
                    c1 = c1 && khi1 == mhi;
                }
                const uint32_t b0 = c0 ? klo0 : CP_NONE, b1 = c1 ? klo1 : CP_NONE;
                const uint32_t mlo = wave_min_u32(b0 < b1 ? b0 : b1);
                const int victim = (POLICY == REMOE_CACHE_BELADY) ? 127 - (int)(mlo & 127u) : (int)(mlo & 127u);
                const unsigned long long keep = ~(1ull << (victim & 63));
                if (victim < 64) { res_lo &= keep; free_lo &= keep; }
                else { res_hi &= keep; free_hi &= keep; }
                --held;
            }
            if (lane == tt) {
                o_miss = (uint32_t)miss;
                o_uniq = (uint32_t)n_u;
                o_hit = (uint32_t)hit_tok;
            }
            total += (unsigned long long)miss;
            total_u += (unsigned long long)n_u;
        }
        if (lane < n) {
            out_miss[s * T + t0 + lane] = (uint8_t)o_miss;
            out_uniq[s * T + t0 + lane] = (uint8_t)o_uniq;
            out_hit_tok[s * T + t0 + lane] = (uint8_t)o_hit;
        }
        __syncthreads();       // the staged rows are replaced next
    }
    if (lane == 0) {
        out_total_miss[s] = total;
        out_total_uniq[s] = total_u;
        out_bytes[s] = total * expert_bytes;
    }
}

// Routing with a residency bonus + LRU, one wavefront per trace.  Score of expert e at step t:
// P_t[e] * factor if e is resident before the step, else P_t[e] (factor = exp(beta): the same order
// as adding beta to the resident experts' logits); ties to the lower id; gate weights are the
// unmodified probabilities of the chosen experts (divided by their sum when renorm).
constexpr int RR_AHEAD = 4;             // probability rows in flight

__global__ __launch_bounds__(64) void reroute_kernel(const float *__restrict__ probs, int64_t T, int N, int K, int C,
                                                     float factor, int renorm, int32_t *__restrict__ out_idx,
                                                     float *__restrict__ out_w, uint8_t *__restrict__ out_miss,
                                                     unsigned long long *__restrict__ out_total_miss)
{
    const int64_t s = blockIdx.x;
    const int lane = threadIdx.x;
    const float *pr = probs + s * T * N;
    const float NEG_INF = -__builtin_inff();
    unsigned long long res_lo = 0ull, res_hi = 0ull;      // resident experts (wave-uniform masks)
    uint32_t key0 = 0, key1 = 0;                          // (step of last use + 1, id) of experts lane, lane + 64
    unsigned long long total = 0;
    float q0[RR_AHEAD], q1[RR_AHEAD];
#pragma unroll
    for (int a = 0; a < RR_AHEAD; ++a) {
        q0[a] = (a < T && lane < N) ? pr[(int64_t)a * N + lane] : 0.f;
        q1[a] = (a < T && lane + 64 < N) ? pr[(int64_t)a * N + lane + 64] : 0.f;
    }
    for (int64_t tb = 0; tb < T; tb += RR_AHEAD) {
#pragma unroll
        for (int a = 0; a < RR_AHEAD; ++a) {
            const int64_t t = tb + a;
            if (t >= T) break;
            const float p0 = q0[a], p1 = q1[a];
            // the row RR_AHEAD steps ahead takes this slot
            const int64_t tn = t + RR_AHEAD;
            q0[a] = (tn < T && lane < N) ? pr[tn * N + lane] : 0.f;
            q1[a] = (tn < T && lane + 64 < N) ? pr[tn * N + lane + 64] : 0.f;

            const bool res0 = ((res_lo >> lane) & 1ull) != 0ull, res1 = ((res_hi >> lane) & 1ull) != 0ull;
            float m0 = lane < N ? (res0 ? p0 * factor : p0) : NEG_INF;
            float m1 = lane + 64 < N ? (res1 ? p1 * factor : p1) : NEG_INF;
            unsigned long long sel_lo = 0ull, sel_hi = 0ull;
            int my_e = 0;
            for (int j = 0; j < K; ++j) {
                const float m = wave_max(fmaxf(m0, m1));
                const unsigned long long b0 = __ballot(m0 == m), b1 = __ballot(m1 == m);
                const int e = b0 ? __ffsll((long long)b0) - 1 : 63 + __ffsll((long long)b1);
                if (lane == j) my_e = e;
                if (e == lane) m0 = NEG_INF;
                if (e == lane + 64) m1 = NEG_INF;
                if (e < 64) sel_lo |= 1ull << e;
                else sel_hi |= 1ull << (e - 64);
            }
            // the unmodified probability of lane j's expert, fetched once for all K places
            const float pe_lo = __shfl(p0, my_e & 63, 64), pe_hi = __shfl(p1, my_e & 63, 64);
            const float my_p = lane < K ? (my_e < 64 ? pe_lo : pe_hi) : 0.f;
            float wgt = my_p;
            if (renorm) wgt = my_p / wave_sum(my_p);
            if (lane < K) {
                out_idx[(s * T + t) * K + lane] = my_e;
                out_w[(s * T + t) * K + lane] = wgt;
            }
            // LRU: misses against the state before the step, then the chosen experts become the most recent
            const int miss = __popcll(sel_lo & ~res_lo) + __popcll(sel_hi & ~res_hi);
            const uint32_t stamp = ((uint32_t)(t + 1) << 7);
            if ((sel_lo >> lane) & 1ull) key0 = stamp | (uint32_t)lane;
            if ((sel_hi >> lane) & 1ull) key1 = stamp | (uint32_t)(lane + 64);
            res_lo |= sel_lo;
            res_hi |= sel_hi;
            int held = __popcll(res_lo) + __popcll(res_hi);
            const int n_sel = __popcll(sel_lo) + __popcll(sel_hi);
            if (n_sel >= C) {
                // the step alone fills the cache (C = 4 under top-6 routing in App. G): everything older goes,
                // and of the step's experts, all equally recent, the C highest ids stay
                res_lo = sel_lo;
                res_hi = sel_hi;
                for (int d = n_sel - C; d > 0; --d) {
                    if (res_lo) res_lo &= res_lo - 1ull;
                    else res_hi &= res_hi - 1ull;
                }
                held = C;
            }
            while (held > C) {
                const uint32_t b0 = ((res_lo >> lane) & 1ull) ? key0 : CP_NONE, b1 = ((res_hi >> lane) & 1ull) ? key1 : CP_NONE;
                const uint32_t mk = wave_min_u32(b0 < b1 ? b0 : b1);     // a key ends in its expert's id
                const int victim = (int)(mk & 127u);
                if (victim < 64) res_lo &= ~(1ull << victim);
                else res_hi &= ~(1ull << (victim - 64));
                --held;
            }
            if (lane == 0) out_miss[s * T + t] = (uint8_t)miss;
            total += (unsigned long long)miss;
        }
    }
    if (lane == 0) out_total_miss[s] = total;
}

// ---- per-step sums over layers, histogram, percentiles -----------------------------------------------
constexpr int SS_MAX_HIST = 4097;       // sums up to 64 layers x 64 experts

__global__ void zero_u64_kernel(unsigned long long *p, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0ull;
}

__global__ __launch_bounds__(256) void step_summary_kernel(const uint8_t *__restrict__ miss, int64_t L, int64_t n,
                                                           uint16_t *__restrict__ out_all,
                                                           unsigned long long *__restrict__ hist, int hist_len)
{
    __shared__ uint32_t lh[SS_MAX_HIST];
    for (int v = threadIdx.x; v < hist_len; v += blockDim.x) lh[v] = 0u;
    __syncthreads();
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        uint32_t a = 0;
        for (int64_t l = 0; l < L; ++l) a += miss[l * n + i];
        out_all[i] = (uint16_t)a;
        atomicAdd(&lh[(int)a < hist_len ? a : (uint32_t)(hist_len - 1)], 1u);   // sums beyond the table share its last bin
    }
    __syncthreads();
    for (int v = threadIdx.x; v < hist_len; v += blockDim.x)
        if (lh[v]) atomicAdd(&hist[v], (unsigned long long)lh[v]);   // integer sums: exact in any order
}

// percentile p = smallest v whose cumulative count reaches p percent of the n steps
__global__ void step_percentile_kernel(const unsigned long long *__restrict__ hist, int hist_len, unsigned long long n,
                                       int32_t *__restrict__ out_pct)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const unsigned long long pcts[3] = {50ull, 95ull, 99ull};
    for (int k = 0; k < 3; ++k) {
        unsigned long long cum = 0;
        int32_t ans = -1;
        for (int v = 0; v < hist_len && ans < 0; ++v) {
            cum += hist[v];
            if (n > 0 && 100ull * cum >= pcts[k] * n) ans = v;
        }
        out_pct[k] = ans;
    }
}

// ---- expert-load balance of a trace -------------------------------------------------------------------
__device__ __forceinline__ double wave_sum_f64(double v)
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

__global__ __launch_bounds__(256) void balance_kernel(const int32_t *__restrict__ idx, int64_t T, int K, int N,
                                                      uint32_t *__restrict__ out_load, int32_t *__restrict__ out_used,
                                                      double *__restrict__ out_entropy, double *__restrict__ out_cv)
{
    __shared__ uint32_t load[128];
    const int64_t s = blockIdx.x;
    if (threadIdx.x < 128) load[threadIdx.x] = 0u;
    __syncthreads();
    const int32_t *tr = idx + s * T * K;
    for (int64_t q = threadIdx.x; q < T * K; q += blockDim.x) {
        const int e = tr[q];
        if (e >= 0 && e < N) atomicAdd(&load[e], 1u);
    }
    __syncthreads();
    if (threadIdx.x < N) out_load[s * N + threadIdx.x] = load[threadIdx.x];
    if (threadIdx.x < 64) {
        const int lane = threadIdx.x;
        const double total = (double)T * (double)K;
        const double m = total / (double)N;
        double h = 0.0, var = 0.0;
        int used = 0;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int e = lane + 64 * half;
            if (e < N) {
                const double c = (double)load[e];
                if (load[e] > 0u) {
                    const double p = c / total;
                    h -= p * log(p);
                }
                var += (c - m) * (c - m);
            }
            used += __popcll(__ballot(e < N && load[e] > 0u));
        }
        h = wave_sum_f64(h);
        var = wave_sum_f64(var);
        if (lane == 0) {
            out_used[s] = used;
            out_entropy[s] = (total > 0.0 && N > 1) ? h / log((double)N) : 0.0;
            out_cv[s] = (total > 0.0) ? sqrt(var / (double)N) / m : 0.0;
        }
    }
}

}  // namespace

size_t cache_workspace_bytes(int64_t S, int64_t T, int K, int policy)
{
    return policy == REMOE_CACHE_BELADY ? align_up(sizeof(int32_t) * (size_t)S * (size_t)T * (size_t)K, 256) : 0;
}

remoe_status launch_cache_policy(const int32_t *idx, int64_t S, int64_t T, int K, int N, int C, int policy,
                                 uint64_t expert_bytes, uint8_t *miss, uint8_t *uniq, uint8_t *hit_tok,
                                 uint64_t *total_miss, uint64_t *total_uniq, uint64_t *bytes, void *workspace,
                                 hipStream_t stream)
{
    if (S == 0) return REMOE_OK;
    const dim3 grid((unsigned)S), block(64);
    unsigned long long *tm = reinterpret_cast<unsigned long long *>(total_miss);
    unsigned long long *tu = reinterpret_cast<unsigned long long *>(total_uniq);
    unsigned long long *tb = reinterpret_cast<unsigned long long *>(bytes);
    int32_t *nxt = static_cast<int32_t *>(workspace);
    switch (policy) {
    case REMOE_CACHE_LRU:
        hipLaunchKernelGGL(cache_policy_kernel<REMOE_CACHE_LRU>, grid, block, 0, stream, idx, T, K, N, C, expert_bytes, nxt, miss,
                           uniq, hit_tok, tm, tu, tb);
        break;
    case REMOE_CACHE_FIFO:
        hipLaunchKernelGGL(cache_policy_kernel<REMOE_CACHE_FIFO>, grid, block, 0, stream, idx, T, K, N, C, expert_bytes, nxt, miss,
                           uniq, hit_tok, tm, tu, tb);
        break;
    case REMOE_CACHE_LFU:
        hipLaunchKernelGGL(cache_policy_kernel<REMOE_CACHE_LFU>, grid, block, 0, stream, idx, T, K, N, C, expert_bytes, nxt, miss,
                           uniq, hit_tok, tm, tu, tb);
        break;
    case REMOE_CACHE_BELADY:
        hipLaunchKernelGGL(next_use_kernel, grid, block, 0, stream, idx, T, K, N, nxt);
        hipLaunchKernelGGL(cache_policy_kernel<REMOE_CACHE_BELADY>, grid, block, 0, stream, idx, T, K, N, C, expert_bytes, nxt,
                           miss, uniq, hit_tok, tm, tu, tb);
        break;
    default:
        return fail(REMOE_E_INVALID_ARG, "unknown cache policy %d", policy);
    }
    return check_hip(hipGetLastError(), "cache_policy_kernel launch");
}

remoe_status launch_reroute(const float *probs, int64_t S, int64_t T, int N, int K, int C, float factor, int renorm,
                            int32_t *idx, float *w, uint8_t *miss, uint64_t *total_miss, hipStream_t stream)
{
    if (S == 0) return REMOE_OK;
    hipLaunchKernelGGL(reroute_kernel, dim3((unsigned)S), dim3(64), 0, stream, probs, T, N, K, C, factor, renorm, idx, w, miss,
                       reinterpret_cast<unsigned long long *>(total_miss));
    return check_hip(hipGetLastError(), "reroute_kernel launch");
}

int step_summary_max_hist() { return SS_MAX_HIST; }

remoe_status launch_step_summary(const uint8_t *miss, int64_t L, int64_t S, int64_t T, uint16_t *out_all,
                                 uint64_t *hist, int hist_len, int32_t *pct, hipStream_t stream)
{
    const int64_t n = S * T;
    unsigned long long *h = reinterpret_cast<unsigned long long *>(hist);
    hipLaunchKernelGGL(zero_u64_kernel, dim3(1), dim3(256), 0, stream, h, (int64_t)hist_len);
    if (n > 0) {
        int64_t blocks = ceil_div(n, 256);
        if (blocks > 2048) blocks = 2048;
        hipLaunchKernelGGL(step_summary_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, miss, L, n, out_all, h, hist_len);
    }
    hipLaunchKernelGGL(step_percentile_kernel, dim3(1), dim3(64), 0, stream, h, hist_len, (unsigned long long)n, pct);
    return check_hip(hipGetLastError(), "step_summary launch");
}

remoe_status launch_balance(const int32_t *idx, int64_t S, int64_t T, int K, int N, uint32_t *load, int32_t *used,
                            double *entropy, double *cv, hipStream_t stream)
{
    if (S == 0) return REMOE_OK;
    hipLaunchKernelGGL(balance_kernel, dim3((unsigned)S), dim3(256), 0, stream, idx, T, K, N, load, used, entropy, cv);
    return check_hip(hipGetLastError(), "balance_kernel launch");
}

}  // namespace remoe
