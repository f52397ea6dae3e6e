// Routing-trace statistics on expert-set bitmasks: adjacent-step overlap and LRU cache misses.
//
// trace_reuse_kernel: |E_t ∩ E_{t-1}|, the numerator of IR_t (Eq. 1).  One workgroup per trace
// (a (sequence, layer) pair); each thread turns two consecutive steps into 128-bit masks and
// counts the bits of their AND.
//
// lru_kernel: the per-layer LRU expert cache of the paper's simulator (App. A cache model,
// App. E.2 unique-miss accounting).  One wavefront per trace; lane l owns experts l and l+64 and
// keeps one recency key per expert, key = ((last step + 1) << 7) | id, 0 = never used.  The
// cache before a step holds the C largest keys, so a requested expert hits iff it was used
// before and fewer than C experts carry a larger key.  The key order (step, then id) makes
// experts of one step age in ascending id order.
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

constexpr int LRU_STAGE_INTS = 4096;  // expert ids staged in LDS per chunk of steps

__global__ __launch_bounds__(64) void lru_kernel(const int32_t *__restrict__ idx, int64_t T, int K,
                                                 int N, int C, unsigned long long expert_bytes,
                                                 int64_t step0, uint32_t *__restrict__ state,
                                                 uint8_t *__restrict__ miss_out,
                                                 uint64_t *__restrict__ total_out,
                                                 uint64_t *__restrict__ bytes_out)
{
    __shared__ int32_t ids[LRU_STAGE_INTS];
    const int64_t s = blockIdx.x;
    const int lane = threadIdx.x;
    const int32_t *tr = idx + s * T * K;

    uint32_t key0 = 0, key1 = 0;
    if (state) {
        const uint32_t l0 = (lane < N) ? state[s * N + lane] : 0u;
        const uint32_t l1 = (lane + 64 < N) ? state[s * N + lane + 64] : 0u;
        key0 = l0 ? ((l0 << 7) | (uint32_t)lane) : 0u;
        key1 = l1 ? ((l1 << 7) | (uint32_t)(lane + 64)) : 0u;
    }

    const int chunk_steps = LRU_STAGE_INTS / K;
    unsigned long long total = 0;
    for (int64_t base = 0; base < T; base += chunk_steps) {
        const int ns = (int)((T - base < chunk_steps) ? (T - base) : chunk_steps);
        __syncthreads();
        for (int q = lane; q < ns * K; q += 64) ids[q] = tr[base * K + q];
        __syncthreads();
        int my_miss = 0;
        for (int tl = 0; tl < ns; ++tl) {
            bool req0 = false, req1 = false;
            for (int j = 0; j < K; ++j) {
                const int e = ids[tl * K + j];   // same address in every lane: LDS broadcast
                req0 |= (e == lane);
                req1 |= (e == lane + 64);
            }
            req0 &= (lane < N);
            req1 &= (lane + 64 < N);
            unsigned long long m0 = __ballot(req0), m1 = __ballot(req1);
            const int n_unique = __popcll(m0) + __popcll(m1);
            int hits = 0;
            while (m0) {
                const int b = __ffsll((long long)m0) - 1;
                m0 &= m0 - 1;
                const uint32_t ke = __shfl(key0, b, 64);
                const int above = __popcll(__ballot(key0 > ke)) + __popcll(__ballot(key1 > ke));
                hits += (ke != 0u && above < C);
            }
            while (m1) {
                const int b = __ffsll((long long)m1) - 1;
                m1 &= m1 - 1;
                const uint32_t ke = __shfl(key1, b, 64);
                const int above = __popcll(__ballot(key0 > ke)) + __popcll(__ballot(key1 > ke));
                hits += (ke != 0u && above < C);
            }
            const int miss = n_unique - hits;
            total += (unsigned long long)miss;
            if ((tl & 63) == lane) my_miss = miss;
            const uint32_t stamp = (uint32_t)(step0 + base + tl + 1) << 7;
            if (req0) key0 = stamp | (uint32_t)lane;
            if (req1) key1 = stamp | (uint32_t)(lane + 64);
            if ((tl & 63) == 63 || tl == ns - 1) {
                const int first = tl & ~63;
                if (first + lane <= tl) miss_out[s * T + base + first + lane] = (uint8_t)my_miss;
            }
        }
    }
    if (state) {
        if (lane < N) state[s * N + lane] = key0 >> 7;
        if (lane + 64 < N) state[s * N + lane + 64] = key1 >> 7;
    }
    if (lane == 0) {
        total_out[s] = total;
        bytes_out[s] = total * expert_bytes;
    }
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
    hipLaunchKernelGGL(lru_kernel, dim3((unsigned)S), dim3(64), 0, stream, idx, T, K, N, C,
                       (unsigned long long)expert_bytes, step0, state, miss, total, bytes);
    return check_hip(hipGetLastError(), "lru_kernel launch");
}

}  // namespace remoe
