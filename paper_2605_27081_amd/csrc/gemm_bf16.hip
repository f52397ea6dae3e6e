// Grouped expert GEMMs on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate).
//
// The selected experts "execute as in the base model" (Sec. 4.1, step 5); with SwiGLU experts that
// is, per expert e and for the rows (token, j) routed to it,
//   mode 0:  h   = silu(X_e W_gate[e]^T) * (X_e W_up[e]^T)          -> [slots, I]   bf16
//   mode 1:  out = (h_e W_down[e]^T) * gate weight of the row       -> [slots, H]   bf16
// Both are C[m, n] = sum_k A[row(m), k] * B_e[n, k] with the reduction dimension contiguous in both
// operands, which is exactly the per-lane operand layout of the 32x32x16 MFMA (8 consecutive k per
// lane), so LDS fragments are single 16-byte reads.
//
// Tiling: 128 x 128 x 64 per workgroup of 4 wavefronts (2 x 2, 64 x 64 each = 2 x 2 MFMA tiles).
// In mode 0 the 128 B-rows are 64 gate rows + the 64 matching up rows, so a lane holds g and u of
// the same (m, n) in two accumulators and applies SwiGLU in registers.  LDS rows are 8 chunks of
// 16 bytes in an XOR-swizzled layout (lds_slot) that keeps the row-per-lane fragment reads and the
// 8-lanes-per-row global->LDS copies free of bank conflicts.  Global loads run two tiles ahead of the
// MFMAs through two register sets and are copied to the other LDS stage after the MFMAs of the
// current tile (one barrier per step).
//
// Rows of A are gathered through slot -> token, so no permuted copy of x is ever materialised.
// The tile list (expert, first slot, valid rows) comes from the permute step and lives in device
// memory; the launch covers an upper bound of tiles and surplus workgroups return at once.
// Workgroup ids are dealt round-robin to the 8 XCDs, so id b works on logical tile
// (b % 8) * chunk + b / 8: every XCD walks one contiguous range (n-tile fastest), which keeps an
// expert's weights and the current A rows hot in that XCD's L2.
#include "common.h"

namespace remoe {

namespace {

constexpr int GM_BM = 128;
constexpr int GM_BK = 64;
constexpr int GM_STAGE = GM_BM * 8;  // 16-byte chunks per operand per stage

// LDS tile layout: rows of 8 chunks (16 bytes each).  Chunk c of row r lives in row slot
// r ^ ((r >> 3) & 1) at chunk position c ^ (r & 7).  A fragment read has lane i on row base+i with
// one logical chunk: any 8 consecutive lanes then hit 8 different chunk positions (all 32 banks of
// a 128-byte period), and rows r, r+8 land in row slots of opposite parity, so 16 consecutive
// lanes also cover a full 256-byte period.  The 8-lanes-per-row copies into LDS stay conflict-free.
__device__ __forceinline__ int lds_slot(int r, int c) { return ((r ^ ((r >> 3) & 1)) << 3) + (c ^ (r & 7)); }

struct KArgs {
    const bf16_t *a;
    int64_t lda;
    const int32_t *row_gather;
    const bf16_t *b0;
    const bf16_t *b1;
    int k_dim;
    int n_out;
    const int32_t *tile_expert, *tile_row0, *tile_rows, *n_tiles;
    int dense_rows;
    const float *row_scale;
    bf16_t *c;
    int64_t ldc;
    int64_t c_row_offset;
};

template <int MODE>
__global__ __launch_bounds__(256, 2) void grouped_gemm_bf16_kernel(const KArgs p)
{
    constexpr int BN_OUT = (MODE == 0) ? 64 : 128;  // output columns per workgroup
    __shared__ u32x4_t lds_a[2][GM_STAGE];
    __shared__ u32x4_t lds_b[2][GM_STAGE];

    const int ntn = p.n_out / BN_OUT;
    const int n_mt = p.tile_expert ? *p.n_tiles : (p.dense_rows + GM_BM - 1) / GM_BM;
    const int nblk = n_mt * ntn;
    const int chunk = (nblk + 7) >> 3;
    const int q = blockIdx.x >> 3;
    if (q >= chunk) return;
    const int logical = (blockIdx.x & 7) * chunk + q;
    if (logical >= nblk) return;
    const int mt = logical / ntn, nt = logical - mt * ntn;

    int expert = 0, row0 = mt * GM_BM, rows = p.dense_rows - row0;
    if (p.tile_expert) {
        expert = p.tile_expert[mt];
        row0 = p.tile_row0[mt];
        rows = p.tile_rows[mt];
    }
    if (rows > GM_BM) rows = GM_BM;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, lh = lane >> 5;
    const int lc = tid & 7;   // 16-byte chunk this thread copies
    const int lr = tid >> 3;  // first of its 4 rows (stride 32)

    const bf16_t *ap[4];
    const bf16_t *bp[4];
    const int64_t estride = (int64_t)p.n_out * p.k_dim;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int r = lr + 32 * i;
        int rr = r < rows ? r : rows - 1;
        int64_t arow = row0 + rr;
        if (p.row_gather) arow = p.row_gather[arow];
        ap[i] = p.a + arow * p.lda + lc * 8;
        if (MODE == 0) {
            const bf16_t *base = (r < 64) ? p.b0 : p.b1;
            bp[i] = base + expert * estride + (int64_t)(nt * 64 + (r & 63)) * p.k_dim + lc * 8;
        } else {
            bp[i] = p.b0 + expert * estride + (int64_t)(nt * 128 + r) * p.k_dim + lc * 8;
        }
    }

    floatx16_t acc[2][2];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

    // Two register sets stage the global loads: while tile k is multiplied out of LDS, tile k+1 is
    // already in (or on its way to) one set and the loads of tile k+2 are issued into the other,
    // so every load has more than a full MFMA phase to arrive before it is copied into LDS.
    u32x4_t ga0[4], gb0[4], ga1[4], gb1[4];
#define GM_LOAD_GLOBAL(ga, gb, k0)                                                      \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                      \
        ga[i] = *reinterpret_cast<const u32x4_t *>(ap[i] + (k0));                        \
        gb[i] = *reinterpret_cast<const u32x4_t *>(bp[i] + (k0));                        \
    }                                                                                   \
    __builtin_amdgcn_sched_barrier(0);   /* keep the loads ahead of the MFMA phase */
#define GM_STORE_LDS(ga, gb, stage)                                                     \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                      \
        const int r_ = lr + 32 * i;                                                     \
        lds_a[stage][lds_slot(r_, lc)] = ga[i];                                         \
        lds_b[stage][lds_slot(r_, lc)] = gb[i];                                         \
    }
    // Fragments are double-buffered in registers: the LDS reads of k-step ks+1 are issued before
    // the four MFMAs of k-step ks, so their latency hides behind matrix-core work.
#define GM_READ_FRAGS(stage, ks, fa, fb)                                                \
    _Pragma("unroll") for (int mi = 0; mi < 2; ++mi)                                     \
        fa[mi] = *reinterpret_cast<const bf16x8_t *>(&lds_a[stage][lds_slot(a_row[mi], 2 * (ks) + lh)]); \
    _Pragma("unroll") for (int ni = 0; ni < 2; ++ni)                                     \
        fb[ni] = *reinterpret_cast<const bf16x8_t *>(&lds_b[stage][lds_slot(b_row[ni], 2 * (ks) + lh)]);
#define GM_MFMA(fa, fb)                                                                 \
    _Pragma("unroll") for (int mi = 0; mi < 2; ++mi)                                     \
        _Pragma("unroll") for (int ni = 0; ni < 2; ++ni)                                 \
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[mi], fb[ni], acc[mi][ni], 0, 0, 0);
#define GM_COMPUTE(stage)                                                               \
    {                                                                                   \
        bf16x8_t fa0[2], fb0[2], fa1[2], fb1[2];                                        \
        GM_READ_FRAGS(stage, 0, fa0, fb0)                                               \
        GM_READ_FRAGS(stage, 1, fa1, fb1)                                               \
        __builtin_amdgcn_sched_barrier(0);                                              \
        GM_MFMA(fa0, fb0)                                                               \
        __builtin_amdgcn_sched_barrier(0);                                              \
        GM_READ_FRAGS(stage, 2, fa0, fb0)                                               \
        __builtin_amdgcn_sched_barrier(0);                                              \
        GM_MFMA(fa1, fb1)                                                               \
        __builtin_amdgcn_sched_barrier(0);                                              \
        GM_READ_FRAGS(stage, 3, fa1, fb1)                                               \
        __builtin_amdgcn_sched_barrier(0);                                              \
        GM_MFMA(fa0, fb0)                                                               \
        __builtin_amdgcn_sched_barrier(0);                                              \
        GM_MFMA(fa1, fb1)                                                               \
    }

    int a_row[2], b_row[2];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi) a_row[mi] = wm * 64 + mi * 32 + li;
    if (MODE == 0) {
        b_row[0] = wn * 32 + li;
        b_row[1] = 64 + wn * 32 + li;
    } else {
        b_row[0] = wn * 64 + li;
        b_row[1] = wn * 64 + 32 + li;
    }

    const int nk = p.k_dim / GM_BK;   // >= 1
    GM_LOAD_GLOBAL(ga0, gb0, 0)
    if (nk > 1) { GM_LOAD_GLOBAL(ga1, gb1, GM_BK) }
    GM_STORE_LDS(ga0, gb0, 0)
    __syncthreads();
    // tile kt sits in LDS stage kt & 1; even kt: set 1 holds tile kt+1, set 0 is free (and vice versa).
    // The steady-state loop issues its loads unconditionally, so the waits before the LDS copies
    // cover only the older set; the last (up to three) tiles run through the guarded copy below.
    int kt = 0;
    for (; kt + 3 < nk; kt += 2) {
        GM_LOAD_GLOBAL(ga0, gb0, (kt + 2) * GM_BK)
        GM_COMPUTE(0)
        GM_STORE_LDS(ga1, gb1, 1)
        __syncthreads();
        GM_LOAD_GLOBAL(ga1, gb1, (kt + 3) * GM_BK)
        GM_COMPUTE(1)
        GM_STORE_LDS(ga0, gb0, 0)
        __syncthreads();
    }
    for (; kt < nk; kt += 2) {
        if (kt + 2 < nk) { GM_LOAD_GLOBAL(ga0, gb0, (kt + 2) * GM_BK) }
        GM_COMPUTE(0)
        if (kt + 1 < nk) { GM_STORE_LDS(ga1, gb1, 1) }
        __syncthreads();
        if (kt + 1 >= nk) break;
        GM_COMPUTE(1)
        if (kt + 2 < nk) { GM_STORE_LDS(ga0, gb0, 0) }
        __syncthreads();
    }

    // epilogue: a lane holds column li of 16 rows per accumulator
#pragma unroll
    for (int mi = 0; mi < 2; ++mi) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = wm * 64 + mi * 32 + (r >> 2) * 8 + lh * 4 + (r & 3);
            if (m >= rows) continue;
            const int64_t crow = (p.c_row_offset + row0 + m) * p.ldc;
            if (MODE == 0) {
                const float g = acc[mi][0][r], u = acc[mi][1][r];
                const float h = g / (1.0f + __expf(-g)) * u;
                p.c[crow + nt * 64 + wn * 32 + li] = f32_to_bf16(h);
            } else {
                const float sc = p.row_scale ? p.row_scale[row0 + m] : 1.0f;
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
                    p.c[crow + nt * 128 + wn * 64 + ni * 32 + li] = f32_to_bf16(acc[mi][ni][r] * sc);
            }
        }
    }
}

}  // namespace

int gemm_tile_m() { return GM_BM; }

remoe_status launch_grouped_gemm_bf16(int mode, const GroupedGemmArgs &g, hipStream_t stream)
{
    const int bn = (mode == 0) ? 64 : 128;
    if (g.k_dim % GM_BK != 0 || g.n_out % bn != 0)
        return fail(REMOE_E_UNSUPPORTED, "bf16 GEMM needs k %% 64 == 0 and n %% %d == 0 (k=%d n=%d)", bn,
                    g.k_dim, g.n_out);
    if (g.max_tiles <= 0) return REMOE_OK;
    KArgs p;
    p.a = static_cast<const bf16_t *>(g.a);
    p.lda = g.lda;
    p.row_gather = g.row_gather;
    p.b0 = static_cast<const bf16_t *>(g.b0);
    p.b1 = static_cast<const bf16_t *>(g.b1);
    p.k_dim = g.k_dim;
    p.n_out = g.n_out;
    p.tile_expert = g.tile_expert;
    p.tile_row0 = g.tile_row0;
    p.tile_rows = g.tile_rows;
    p.n_tiles = g.n_tiles;
    p.dense_rows = (int)g.dense_rows;
    p.row_scale = g.row_scale;
    p.c = static_cast<bf16_t *>(g.c);
    p.ldc = g.ldc;
    p.c_row_offset = g.c_row_offset;
    const int64_t nblk = (int64_t)g.max_tiles * (g.n_out / bn);
    const dim3 grid((unsigned)(ceil_div(nblk, 8) * 8)), block(256);
    if (mode == 0)
        hipLaunchKernelGGL(grouped_gemm_bf16_kernel<0>, grid, block, 0, stream, p);
    else
        hipLaunchKernelGGL(grouped_gemm_bf16_kernel<1>, grid, block, 0, stream, p);
    return check_hip(hipGetLastError(), "grouped_gemm_bf16 launch");
}

}  // namespace remoe
