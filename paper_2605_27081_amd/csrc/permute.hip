// Token -> expert counting sort ("permute") and the tile map of the grouped GEMMs.
//
// The routed experts execute on the rows assigned to them (Sec. 4.1, step 5), so the T*K
// (token, j) pairs are sorted by expert id.  The sort is stable (tokens stay in increasing order
// inside an expert) and free of atomics on global memory, hence deterministic:
//   1. permute_count : per workgroup of 256 tokens, an LDS bit matrix [expert][token] gives each
//                      pair its rank among the workgroup's pairs of the same expert, plus the
//                      workgroup's expert histogram;
//   2. permute_scan  : one workgroup turns the histograms into per-workgroup offsets, the
//                      exclusive prefix sum over experts and the list of GEMM row tiles;
//   3. permute_place : slot = offset[expert] + block offset + rank; writes slot -> token,
//                      slot -> gate weight and pair -> slot.
#include "common.h"

namespace remoe {

namespace {

constexpr int PM_TOKENS = 256;  // tokens per workgroup in steps 1 and 3

__global__ __launch_bounds__(PM_TOKENS) void permute_count(const int32_t *__restrict__ idx, int64_t T,
                                                           int K, int N,
                                                           int32_t *__restrict__ blk_hist,
                                                           int32_t *__restrict__ pair_rank)
{
    __shared__ uint32_t bits[128][PM_TOKENS / 32];
    const int tid = threadIdx.x;
    for (int q = tid; q < 128 * (PM_TOKENS / 32); q += PM_TOKENS) (&bits[0][0])[q] = 0u;
    __syncthreads();
    const int64_t t = (int64_t)blockIdx.x * PM_TOKENS + tid;
    const int word = tid >> 5;
    const uint32_t bit = 1u << (tid & 31);
    if (t < T)
        for (int j = 0; j < K; ++j) atomicOr(&bits[idx[t * K + j]][word], bit);
    __syncthreads();
    if (t < T)
        for (int j = 0; j < K; ++j) {
            const int e = idx[t * K + j];
            int rank = __popc(bits[e][word] & (bit - 1u));
            for (int w = 0; w < word; ++w) rank += __popc(bits[e][w]);
            pair_rank[t * K + j] = rank;
        }
    if (tid < N) {
        int c = 0;
#pragma unroll
        for (int w = 0; w < PM_TOKENS / 32; ++w) c += __popc(bits[tid][w]);
        blk_hist[(int64_t)blockIdx.x * N + tid] = c;
    }
}

// One workgroup of PS_SEG x 128 threads: thread (seg, e) owns expert e's counts of one segment of the
// token blocks, so the running sums over the blocks are PS_SEG times shorter chains of loads.
constexpr int PS_SEG = 8;
__global__ __launch_bounds__(PS_SEG * 128) void permute_scan(const int32_t *__restrict__ blk_hist, int n_blk,
                                                    int N, int tile_m, int max_tiles,
                                                    int32_t *__restrict__ blk_off,
                                                    int32_t *__restrict__ offsets,
                                                    int32_t *__restrict__ tile_expert,
                                                    int32_t *__restrict__ tile_row0,
                                                    int32_t *__restrict__ tile_rows,
                                                    int32_t *__restrict__ n_tiles, uint32_t *__restrict__ gemm_ctr)
{
    __shared__ int32_t cnt[128], off[129], tstart[129], seg_sum[PS_SEG][128];
    const int e = threadIdx.x & 127, seg = threadIdx.x >> 7;
    if (threadIdx.x < GEMM_CTR_SETS * 8) gemm_ctr[threadIdx.x] = 0u;   // tile counters of the GEMM launches that follow
    const int per_seg = (n_blk + PS_SEG - 1) / PS_SEG;
    const int b0 = seg * per_seg, b1 = (b0 + per_seg < n_blk) ? b0 + per_seg : n_blk;
    int sum = 0;
    if (e < N) {
#pragma unroll 8
        for (int b = b0; b < b1; ++b) sum += blk_hist[(int64_t)b * N + e];
    }
    seg_sum[seg][e] = sum;
    __syncthreads();
    int run = 0;
    for (int q = 0; q < seg; ++q) run += seg_sum[q][e];
    if (e < N) {
#pragma unroll 8
        for (int b = b0; b < b1; ++b) {
            const int c = blk_hist[(int64_t)b * N + e];
            blk_off[(int64_t)b * N + e] = run;
            run += c;
        }
    }
    if (seg == PS_SEG - 1) cnt[e] = (e < N) ? run : 0;   // the last segment ends with the expert's total
    __syncthreads();
    if (threadIdx.x == 0) {
        int o = 0, ts = 0;
        for (int q = 0; q < N; ++q) {
            off[q] = o;
            tstart[q] = ts;
            o += cnt[q];
            ts += (cnt[q] + tile_m - 1) / tile_m;
        }
        off[N] = o;
        tstart[N] = ts;
        *n_tiles = ts < max_tiles ? ts : max_tiles;
    }
    __syncthreads();
    if (seg == 0 && e <= N) offsets[e] = off[e];
    if (threadIdx.x == 0 && N == 128) offsets[128] = off[128];
    if (seg == 0 && e < N) {
        const int nt = tstart[e + 1] - tstart[e];
        for (int i = 0; i < nt; ++i) {
            const int ti = tstart[e] + i;
            if (ti < max_tiles) {
                tile_expert[ti] = e;
                tile_row0[ti] = off[e] + i * tile_m;
                const int left = cnt[e] - i * tile_m;
                tile_rows[ti] = left < tile_m ? left : tile_m;
            }
        }
    }
}

__global__ __launch_bounds__(256) void permute_place(const int32_t *__restrict__ idx,
                                                     const float *__restrict__ w, int64_t n_pairs,
                                                     int K, int N,
                                                     const int32_t *__restrict__ blk_off,
                                                     const int32_t *__restrict__ offsets,
                                                     int32_t *__restrict__ pair_slot,
                                                     int32_t *__restrict__ slot_token,
                                                     float *__restrict__ slot_w)
{
    const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (p >= n_pairs) return;
    const int64_t t = p / K;
    const int e = idx[p];
    const int slot = offsets[e] + blk_off[(t / PM_TOKENS) * N + e] + pair_slot[p];
    pair_slot[p] = slot;
    slot_token[slot] = (int32_t)t;
    slot_w[slot] = w[p];
}

}  // namespace

int permute_tokens_per_block() { return PM_TOKENS; }

remoe_status launch_permute(const int32_t *idx, const float *w, int64_t T, int K, int N,
                            int tile_m, int max_tiles, const PermuteBuffers &pb, hipStream_t stream)
{
    if (T == 0) return REMOE_OK;
    const int n_blk = (int)ceil_div(T, PM_TOKENS);
    int32_t *blk_hist = pb.blk_hist;
    int32_t *blk_off = pb.blk_hist + (int64_t)n_blk * N;
    hipLaunchKernelGGL(permute_count, dim3(n_blk), dim3(PM_TOKENS), 0, stream, idx, T, K, N, blk_hist,
                       pb.pair_slot);
    hipLaunchKernelGGL(permute_scan, dim3(1), dim3(PS_SEG * 128), 0, stream, blk_hist, n_blk, N, tile_m,
                       max_tiles, blk_off, pb.offsets, pb.tile_expert, pb.tile_row0, pb.tile_rows,
                       pb.n_tiles, pb.gemm_ctr);
    const int64_t n_pairs = T * K;
    hipLaunchKernelGGL(permute_place, dim3((unsigned)ceil_div(n_pairs, 256)), dim3(256), 0, stream, idx,
                       w, n_pairs, K, N, blk_off, pb.offsets, pb.pair_slot, pb.slot_token, pb.slot_w);
    return check_hip(hipGetLastError(), "permute launch");
}

}  // namespace remoe
