// Routing-trace statistics on expert-set bitmasks: adjacent-step overlap and LRU cache misses.
//
// trace_reuse_kernel: |E_t ∩ E_{t-1}|, the numerator of IR_t (Eq. 1).  One workgroup per trace
// (a (sequence, layer) pair); each thread turns two consecutive steps into 128-bit masks and
// counts the bits of their AND.
//
// lru_walk_kernel: the per-layer LRU expert cache of the paper's simulator (App. A cache model,
// App. E.2 unique-miss accounting), one thread per step (see below).
#include "common.h"

namespace remoe {

namespace {

__global__ __launch_bounds__(256) void trace_reuse_kernel(const int32_t *__restrict__ idx, int64_t T,
                                                          int K, int N, uint8_t *__restrict__ ov,
                                                          uint64_t *__restrict__ sum)
{
    const int64_t s = blockIdx.x;
    const int32_t *tr = idx + s * T * K;
    unsigned long long local = 0;
    for (int64_t t = threadIdx.x; t < T; t += blockDim.x) {
        unsigned long long c0 = 0, c1 = 0, p0 = 0, p1 = 0;
        for (int j = 0; j < K; ++j) {
            const int e = tr[t * K + j];
            if (e >= 0 && e < N) {
                if (e < 64) c0 |= 1ull << e; else c1 |= 1ull << (e - 64);
            }
        }
        int o = 0;
        if (t > 0) {
            for (int j = 0; j < K; ++j) {
                const int e = tr[(t - 1) * K + j];
                if (e >= 0 && e < N) {
                    if (e < 64) p0 |= 1ull << e; else p1 |= 1ull << (e - 64);
                }
            }
            o = __popcll(c0 & p0) + __popcll(c1 & p1);
        }
        ov[s * T + t] = (uint8_t)o;
        local += (unsigned long long)o;
    }
    // workgroup reduction of the per-thread sums (integer: exact and order independent)
    __shared__ unsigned long long part[4];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const unsigned lo = __shfl_xor((unsigned)(local & 0xFFFFFFFFull), off, 64);
        const unsigned hi = __shfl_xor((unsigned)(local >> 32), off, 64);
        local += ((unsigned long long)hi << 32) | lo;
    }
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = local;
    __syncthreads();
    if (threadIdx.x == 0) sum[s] = part[0] + part[1] + part[2] + part[3];
}

// ---- LRU misses, every step in parallel
//
// With recency keys (step, id) the cache before step t holds the C distinct experts of largest
// key.  Walking back from step t-1 and collecting unseen experts, each step's from the highest id
// down, visits the experts in exactly that key order, so the first C collected are the resident
// set; the walk also ends as soon as every expert of step t has been collected (all hits) or the
// trace, and then the caller's prior state, is exhausted.  Each step of a trace is therefore an
// independent piece of work: one thread per step, 256 consecutive steps per workgroup, with the
// 128-bit masks of those steps and of the 256 before them staged in LDS.  A walk is short when
// the trace keeps touching new experts and, summed over a trace, never longer than N_r passes.
constexpr int LRU_CHUNK = 256;   // steps per workgroup
constexpr int LRU_HALO = 256;    // earlier steps whose masks are staged as well

__device__ __forceinline__ void step_mask(const int32_t *__restrict__ row, int K, int N,
                                          unsigned long long &lo, unsigned long long &hi)
{
    lo = 0;
    hi = 0;
    for (int j = 0; j < K; ++j) {
        const int e = row[j];
        if (e >= 0 && e < N) {
            if (e < 64) lo |= 1ull << e; else hi |= 1ull << (e - 64);
        }
    }
}

__global__ __launch_bounds__(256) void lru_zero_kernel(uint64_t *__restrict__ total, uint64_t *__restrict__ bytes, int64_t S)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < S) { total[i] = 0; bytes[i] = 0; }
}

__global__ __launch_bounds__(LRU_CHUNK) void lru_walk_kernel(const int32_t *__restrict__ idx, int64_t T, int K,
                                                             int N, int C, unsigned long long expert_bytes,
                                                             const uint32_t *__restrict__ state, int n_chunks,
                                                             uint8_t *__restrict__ miss_out,
                                                             unsigned long long *__restrict__ total_out,
                                                             unsigned long long *__restrict__ bytes_out)
{
    __shared__ unsigned long long m_lo[LRU_CHUNK + LRU_HALO], m_hi[LRU_CHUNK + LRU_HALO];
    __shared__ uint32_t prev_key[128];
    __shared__ uint8_t prev_order[128];   // experts of the prior state, most recent first
    __shared__ int n_prev;
    __shared__ unsigned int block_miss;

    const int64_t s = blockIdx.x / n_chunks;
    const int64_t t0 = (int64_t)(blockIdx.x % n_chunks) * LRU_CHUNK;
    const int tid = threadIdx.x;
    const int32_t *tr = idx + s * T * K;

    const int64_t staged0 = t0 > LRU_HALO ? t0 - LRU_HALO : 0;
    for (int i = tid; i < LRU_CHUNK + LRU_HALO; i += LRU_CHUNK) {
        const int64_t u = staged0 + i;
        unsigned long long lo = 0, hi = 0;
        if (u < T && u < t0 + LRU_CHUNK) step_mask(tr + u * K, K, N, lo, hi);
        m_lo[i] = lo;
        m_hi[i] = hi;
    }
    if (tid == 0) { n_prev = 0; block_miss = 0; }
    if (state && tid < 128) {
        const uint32_t l = (tid < N) ? state[s * N + tid] : 0u;
        prev_key[tid] = l ? ((l << 7) | (uint32_t)tid) : 0u;
    }
    __syncthreads();
    if (state && tid < 128) {
        const uint32_t k = prev_key[tid];
        if (k) {
            int above = 0;
            for (int e = 0; e < 128; ++e) above += prev_key[e] > k;
            prev_order[above] = (uint8_t)tid;   // nonzero keys are distinct: the ranks are a permutation
            atomicAdd(&n_prev, 1);
        }
    }
    __syncthreads();

    const int64_t t = t0 + tid;
    int miss = 0;
    if (t < T) {
        const unsigned long long wl = m_lo[t - staged0], wh = m_hi[t - staged0];
        unsigned long long sl = 0, sh = 0;
        int cnt = 0;
        int64_t u = t - 1;
        while (u >= 0 && cnt < C && ((wl & ~sl) | (wh & ~sh))) {
            unsigned long long ml, mh;
            if (u >= staged0) {
                ml = m_lo[u - staged0];
                mh = m_hi[u - staged0];
            } else {
                step_mask(tr + u * K, K, N, ml, mh);
            }
            unsigned long long nl = ml & ~sl, nh = mh & ~sh;
            int c = __popcll(nl) + __popcll(nh);
            const int room = C - cnt;
            while (c > room) {   // the cut falls inside this step: its lowest ids were touched first
                if (nl) nl &= nl - 1; else nh &= nh - 1;
                --c;
            }
            sl |= nl;
            sh |= nh;
            cnt += c;
            --u;
        }
        if (state && u < 0) {
            const int np = n_prev;
            for (int j = 0; j < np && cnt < C && ((wl & ~sl) | (wh & ~sh)); ++j) {
                const int e = prev_order[j];
                const unsigned long long bl = e < 64 ? 1ull << e : 0ull, bh = e < 64 ? 0ull : 1ull << (e - 64);
                if (!((sl & bl) | (sh & bh))) {
                    sl |= bl;
                    sh |= bh;
                    ++cnt;
                }
            }
        }
        miss = __popcll(wl & ~sl) + __popcll(wh & ~sh);
        miss_out[s * T + t] = (uint8_t)miss;
    }
    // integer sums: exact and independent of the order in which workgroups add
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) miss += __shfl_xor(miss, off, 64);
    if ((tid & 63) == 0 && miss) atomicAdd(&block_miss, (unsigned int)miss);
    __syncthreads();
    if (tid == 0 && block_miss) {
        atomicAdd(&total_out[s], (unsigned long long)block_miss);
        atomicAdd(&bytes_out[s], (unsigned long long)block_miss * expert_bytes);
    }
}

// state[e] = (global step of e's last use) + 1 after the call; one workgroup per trace
__global__ __launch_bounds__(256) void lru_state_kernel(const int32_t *__restrict__ idx, int64_t T, int K,
                                                        int N, int64_t step0, uint32_t *__restrict__ state)
{
    __shared__ uint32_t last[128];
    const int64_t s = blockIdx.x;
    const int tid = threadIdx.x;
    if (tid < 128) last[tid] = (tid < N) ? state[s * N + tid] : 0u;
    __syncthreads();
    const int32_t *tr = idx + s * T * K;
    for (int64_t t = tid; t < T; t += blockDim.x) {
        for (int j = 0; j < K; ++j) {
            const int e = tr[t * K + j];
            if (e >= 0 && e < N) atomicMax(&last[e], (uint32_t)(step0 + t + 1));
        }
    }
    __syncthreads();
    if (tid < N) state[s * N + tid] = last[tid];
}

}  // namespace

remoe_status launch_trace_reuse(const int32_t *idx, int64_t S, int64_t T, int K, int N,
                                uint8_t *ov, uint64_t *sum, hipStream_t stream)
{
    if (S == 0) return REMOE_OK;
    hipLaunchKernelGGL(trace_reuse_kernel, dim3((unsigned)S), dim3(256), 0, stream, idx, T, K, N, ov, sum);
    return check_hip(hipGetLastError(), "trace_reuse_kernel launch");
}

remoe_status launch_lru(const int32_t *idx, int64_t S, int64_t T, int K, int N, int C,
                        uint64_t expert_bytes, int64_t step0, uint32_t *state, uint8_t *miss,
                        uint64_t *total, uint64_t *bytes, hipStream_t stream)
{
    if (S == 0) return REMOE_OK;
    hipLaunchKernelGGL(lru_zero_kernel, dim3((unsigned)ceil_div(S, 256)), dim3(256), 0, stream, total, bytes, S);
    REMOE_HIP_TRY(hipGetLastError());
    if (T == 0) return REMOE_OK;
    const int64_t n_chunks = ceil_div(T, LRU_CHUNK);
    if (S * n_chunks >= ((int64_t)1 << 31))
        return fail(REMOE_E_UNSUPPORTED, "lru_simulate: %lld traces x %lld steps exceed one launch", (long long)S, (long long)T);
    hipLaunchKernelGGL(lru_walk_kernel, dim3((unsigned)(S * n_chunks)), dim3(LRU_CHUNK), 0, stream, idx, T, K, N, C,
                       (unsigned long long)expert_bytes, state, (int)n_chunks, miss,
                       reinterpret_cast<unsigned long long *>(total), reinterpret_cast<unsigned long long *>(bytes));
    REMOE_HIP_TRY(hipGetLastError());
    if (state) {   // after every walk has read the prior state
        hipLaunchKernelGGL(lru_state_kernel, dim3((unsigned)S), dim3(256), 0, stream, idx, T, K, N, step0, state);
        REMOE_HIP_TRY(hipGetLastError());
    }
    return REMOE_OK;
}

}  // namespace remoe
