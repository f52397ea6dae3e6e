// Shared host/device helpers of the HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "remoe.h"
#include "remoe_bench.h"

namespace remoe {

typedef unsigned short bf16_t;  // storage of one bfloat16

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float floatx16_t;
typedef __attribute__((ext_vector_type(4))) float floatx4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;  // 16 bytes moved as one register quad

// ---- host-side error reporting ---------------------------------------------------------------
void set_error(const char *fmt, ...);
remoe_status fail(remoe_status code, const char *fmt, ...);
remoe_status check_hip(hipError_t e, const char *what);

#define REMOE_HIP_TRY(expr)                                            \
    do {                                                               \
        remoe_status st__ = ::remoe::check_hip((expr), #expr);         \
        if (st__ != REMOE_OK) return st__;                             \
    } while (0)

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- device helpers ------------------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// round-to-nearest-even; inputs here are finite
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
#if defined(__HIP_DEVICE_COMPILE__)
    // one v_cvt_pk_bf16_f32 on gfx950 (round-to-nearest-even)
    typedef __attribute__((ext_vector_type(2))) float f32x2_;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_;
    const f32x2_ v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_));
#else
    return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
#endif
}

// value held by the neighbouring lane (lane ^ 1), as a DPP quad permute: no LDS traffic
__device__ __forceinline__ float swap_with_neighbour(float v)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0xB1, 0xF, 0xF, true));
#else
    return v;
#endif
}

// ---- kernel launchers (one per source file) -------------------------------------------------
// Router: logits, top-k, softmax weights.  x_dtype as remoe_dtype.
remoe_status launch_route(const void *x, int x_dtype, int64_t T, int H, const float *w_router,
                          int N, int K, int renorm, int32_t *out_idx, float *out_w,
                          float *out_margin, float *out_probs, hipStream_t stream);

// Token -> expert counting sort and tile map.
struct PermuteBuffers {
    int32_t *blk_hist;     // [n_blk, N]   per-block expert counts, then per-block offsets
    int32_t *offsets;      // [N + 1]      first slot of each expert
    int32_t *tile_expert;  // [max_tiles]
    int32_t *tile_row0;    // [max_tiles]  first slot of the tile
    int32_t *tile_rows;    // [max_tiles]  valid rows in the tile
    int32_t *n_tiles;      // [1]
    int32_t *pair_slot;    // [T*K]        (token, j) -> slot
    int32_t *slot_token;   // [T*K]        slot -> token
    float *slot_w;         // [T*K]        slot -> gate weight
    uint32_t *gemm_ctr;    // [GEMM_CTR_SETS * 8] tile counters of the layer's GEMM launches, zeroed by the permute step
};
constexpr int GEMM_CTR_SETS = 4;
int permute_tokens_per_block();
remoe_status launch_permute(const int32_t *idx, const float *w, int64_t T, int K, int N,
                            int tile_m, int max_tiles, const PermuteBuffers &pb, hipStream_t stream);

// Grouped expert GEMMs.  mode 0: gate/up + SwiGLU, mode 1: down projection scaled per row.
struct GroupedGemmArgs {
    const void *a;            // activations [a_rows, lda]
    int64_t lda;
    int64_t a_rows;           // rows of a (bounds the gathered row indices)
    const int32_t *row_gather;  // slot -> row of a, or NULL (row = slot)
    const void *b0;           // mode 0: W_gate, mode 1: W_down   [E, n_out, k_dim]
    const void *b1;           // mode 0: W_up
    int k_dim;                // reduction length
    int n_out;                // output columns
    const int32_t *tile_expert, *tile_row0, *tile_rows, *n_tiles;  // NULL => dense, single group
    int64_t dense_rows;       // rows when dense
    int max_tiles;            // m-tiles launched
    const float *row_scale;   // mode 1: per output row factor, or NULL
    void *c;                  // output [rows, ldc]
    int64_t ldc;
    int64_t c_row_offset;     // added to the output row index
    uint32_t *tile_ctr;       // bf16 kernel: 8 tile counters (one per XCD), zero when the launch starts
};
int gemm_tile_m();
remoe_status launch_grouped_gemm_bf16(int mode, const GroupedGemmArgs &g, hipStream_t stream);
remoe_status launch_grouped_gemm_f32(int mode, const GroupedGemmArgs &g, hipStream_t stream);

// y[t] = sum_j rows[pair_slot[t*K+j]] + s_t * rows[shared_row0 + t]
remoe_status launch_combine(int dtype, const void *rows, const int32_t *pair_slot, const float *pair_w, int64_t T, int K,
                            int H, int64_t shared_row0, int has_shared, const void *x,
                            const float *ws_scale, void *y, hipStream_t stream);

// M = 1 decode over all layers and a range of steps (persistent kernel, one workgroup per compute unit).
struct DecodeLaunch {
    const void *const *layers;   // device [L][4]: w_router, w_gate, w_up, w_down
    const void *x;
    int64_t steps_total, step0, n_steps;
    int n_layers, H, N, I, K, renorm;
    void *y;
    int32_t *out_idx;
    float *out_w;
    int n_caps;
    int caps[4];
    uint64_t expert_bytes;
    uint32_t *lru_state;
    uint8_t *out_overlap, *out_miss;
    uint64_t *sum_overlap, *total_miss, *bytes_fetched;
    void *workspace;
    uint64_t spin_limit_ticks;
};
size_t decode_workspace_bytes(int H, int N, int I, int K);
remoe_status launch_decode(const DecodeLaunch &d, hipStream_t stream);             // layers chained
remoe_status launch_decode_pipelined(const DecodeLaunch &d, hipStream_t stream);   // layers of a step overlapped

// Trace statistics.
remoe_status launch_trace_reuse(const int32_t *idx, int64_t S, int64_t T, int K, int N,
                                uint8_t *ov, uint64_t *sum, hipStream_t stream);
remoe_status launch_lru(const int32_t *idx, int64_t S, int64_t T, int K, int N, int C,
                        uint64_t expert_bytes, int64_t step0, uint32_t *state, uint8_t *miss,
                        uint64_t *total, uint64_t *bytes, hipStream_t stream);

// Cache policies beyond LRU, per-step sums over layers, routing balance.
size_t cache_workspace_bytes(int64_t S, int64_t T, int K, int policy);
remoe_status launch_cache_policy(const int32_t *idx, int64_t S, int64_t T, int K, int N, int C, int policy,
                                 uint64_t expert_bytes, uint8_t *miss, uint8_t *uniq, uint8_t *hit_tok,
                                 uint64_t *total_miss, uint64_t *total_uniq, uint64_t *bytes, void *workspace,
                                 hipStream_t stream);
remoe_status launch_reroute(const float *probs, int64_t S, int64_t T, int N, int K, int C, float factor, int renorm,
                            int32_t *idx, float *w, uint8_t *miss, uint64_t *total_miss, hipStream_t stream);
int step_summary_max_hist();
remoe_status launch_step_summary(const uint8_t *miss, int64_t L, int64_t S, int64_t T, uint16_t *out_all,
                                 uint64_t *hist, int hist_len, int32_t *pct, hipStream_t stream);
remoe_status launch_balance(const int32_t *idx, int64_t S, int64_t T, int K, int N, uint32_t *load, int32_t *used,
                            double *entropy, double *cv, hipStream_t stream);

// ReMoE's router regularisers, forward values.
size_t loss_workspace_bytes(int64_t S);
remoe_status launch_loss_forward(const float *probs, const float *probs_ref, const int32_t *idx, int64_t S, int64_t T,
                                 int N, int K, const int32_t *lags, int n_lags, int window, double *out, void *workspace,
                                 hipStream_t stream);

// Gradient of the regularisers with respect to the router logits; gate gradient dz^T x.
size_t loss_backward_workspace_bytes(int64_t S, int64_t T, int N, int window);
remoe_status launch_loss_backward(const float *probs, const float *probs_ref, const int32_t *idx, int64_t S, int64_t T,
                                  int N, int K, const int32_t *lags, int n_lags, int window, const double *coef,
                                  const double *loss_values, float *dlogits, void *workspace, hipStream_t stream);
size_t gate_grad_workspace_bytes(int64_t T, int N, int H);
remoe_status launch_gate_grad(const float *dz, const void *x, int x_dtype, int64_t T, int N, int H, float *dw, void *workspace,
                              hipStream_t stream);

// Plain copy of known size (yardstick for hardware byte counters).
remoe_status launch_copy_probe(void *dst, const void *src, size_t bytes, hipStream_t stream);

}  // namespace remoe
