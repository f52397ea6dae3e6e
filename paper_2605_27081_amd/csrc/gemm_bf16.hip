// Grouped expert GEMMs on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate).
//
// The selected experts "execute as in the base model" (Sec. 4.1, step 5); with SwiGLU experts that
// is, per expert e and for the rows (token, j) routed to it,
//   mode 0:  h   = silu(X_e W_gate[e]^T) * (X_e W_up[e]^T)          -> [slots, I]   bf16
//   mode 1:  out = h_e W_down[e]^T                                  -> [slots, H]   bf16
// (the gate weight P_t[e] of a row is applied by the combine step, which reads it anyway).
// Both are C[m, n] = sum_k A[row(m), k] * B_e[n, k] with the reduction dimension contiguous in both
// operands, which is exactly the per-lane operand layout of the 32x32x16 MFMA (8 consecutive k per
// lane), so LDS fragments are single 16-byte reads.
//
// Tiling: one workgroup of 8 wavefronts (2 x 4) owns a 256 x 256 x 64 tile; a wavefront owns
// 128 x 64 of it as 4 x 2 MFMA tiles (128 accumulator registers).  The large tile is what keeps the
// kernel off the L2 -> CU bandwidth limit: each 64-deep slice costs 64 KB of loads for 8.4 MFLOP.
// In mode 0 the 256 B-rows are 128 gate rows + the 128 matching up rows, so a lane holds g and u of
// the same (m, n) in two accumulators and applies SwiGLU in registers.  LDS rows are 8 chunks of
// 16 bytes in an XOR-swizzled layout (lds_slot) that keeps the row-per-lane fragment reads and the
// global->LDS copies free of bank conflicts.  Slices move global -> LDS directly
// (global_load_lds_dwordx4, no staging registers) into two stages: a stage is refilled with the slice
// after next as soon as all its fragments have been read, the copy instructions dealt out between
// the MFMAs of the slice's last two k-steps, and has about a slice and a half of MFMA time to land
// (two barriers per slice).  MFMA fragments go through three register buffers, read one to two
// k-steps ahead, so LDS latency hides behind matrix-core work.
// The MFMAs take the B rows as their first operand, so the accumulators hold the tile transposed:
// a lane owns one output row and four adjacent columns per register group, which the epilogue packs
// into 8-byte pieces of a row without exchanging values between lanes.
//
// Rows of A are gathered through slot -> token, so no permuted copy of x is ever materialised.
// The tile list (expert, first slot, valid rows) comes from the permute step and lives in device
// memory; the launch covers an upper bound of tiles and surplus workgroups return at once.
// Workgroup ids are dealt round-robin to the 8 XCDs; every XCD hands out one contiguous range of
// logical tiles to its workgroups in arrival order, which keeps an expert's weights and the current
// A rows hot in that XCD's L2.
#include "common.h"

namespace remoe {

namespace {

constexpr int GM_BK = 64;
// Order of the logical tiles: MT_GROUP row tiles walk the column tiles together, row tile fastest, so
// that workgroups that start one after the other share a weight tile and meet the same row tile
// again MT_GROUP tiles later.  Measured on the Qwen3-shaped layer (65,536 tokens): 4 for gate/up and
// 5 for the down projection (2.85 -> 2.82 ms and 1.82 -> 1.65 ms against column tile fastest; 7 is as
// good as 5, the even sizes 6 and 8 are 2 % and 5 % slower).
constexpr int MT_GROUP0 = 4, MT_GROUP1 = 5;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;   // four bf16 of one output row

// LDS tile layout: rows of 8 chunks (16 bytes each).  Chunk c of row r lives in row slot
// r ^ ((r >> 3) & 1) at chunk position c ^ (r & 7).  A fragment read has lane i on row base+i with
// one logical chunk: any 8 consecutive lanes then hit 8 different chunk positions (all 32 banks of
// a 128-byte period), and rows r, r+8 land in row slots of opposite parity, so 16 consecutive
// lanes also cover a full 256-byte period.  The 8-lanes-per-row copies into LDS stay conflict-free.
__device__ __forceinline__ int lds_slot(int r, int c) { return ((r ^ ((r >> 3) & 1)) << 3) + (c ^ (r & 7)); }

// 64 lanes x 16 bytes, global -> LDS without passing through registers: lane l's 16 bytes, read from
// base + off (wave-uniform 64-bit base, per-lane 32-bit byte offset), land at lds_base + 16 l
// (lds_base wave-uniform, handed over in M0).  Written as assembly so that the compiler keeps no
// books on these copies: its own bookkeeping makes every later LDS read wait for all of them,
// which would undo the overlap.  Every wait for a copy in this file is therefore explicit.
// The compiler pads its own instructions with the wait states the hardware asks for but does not
// look inside an assembly block, so the block must not depend on any:
//   * the address goes in as a per-lane 64-bit value in vector registers (the compiler's own add of
//     base and offset in front of the block).  With the base in a scalar register pair the copy
//     would read a scalar register as a memory address, and a scalar register that a vector
//     instruction has just written (a spilled base restored with v_readlane) may not be used that
//     way for five wait states: whether that happened would depend on register allocation;
//   * M0 is written inside the block and the one wait state the copy needs behind that write is
//     part of the block.  Nothing else in this kernel touches M0 (the compiler reserves it and has
//     no use for it here; a host-side test of the generated code checks that).
__device__ __forceinline__ void copy16_to_lds(const char *base, uint32_t off, const void *lds_base)
{
#if defined(__HIP_DEVICE_COMPILE__)
    const uint32_t dst = (uint32_t)(uintptr_t)lds_base;   // the low 32 bits of a generic LDS pointer are the LDS offset
    const char *src = base + off;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(dst), "v"(src) : "memory");
#else
    (void)base;
    (void)off;
    (void)lds_base;
#endif
}

// Entry idx of a list that no kernel writes while this one runs (the tile list of the permute step),
// fetched through the constant address space: a scalar load, which neither occupies the vector
// memory queue nor has to wait for the stores queued in it.
__device__ __forceinline__ int list_entry(const int32_t *list, int idx)
{
    typedef const int32_t __attribute__((address_space(4))) *const_i32_ptr;
    return *(const_i32_ptr)(uintptr_t)(list + idx);
}

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
    bf16_t *c;
    int64_t ldc;
    int64_t c_row_offset;
    uint32_t *tile_ctr;          // [8] next unclaimed tile of each XCD's range, zero at launch
};

// Claims the next logical tile for a workgroup of XCD `home`: first from that XCD's own contiguous
// range, and once that is used up from the ranges of the other XCDs, so that compute units that run
// ahead (the XCDs do not all stream at the same speed) take over work instead of idling at the end
// of the launch.  Returns -1 when every range is exhausted.
__device__ __forceinline__ int claim_tile(uint32_t *ctr, int home, int chunk, int nblk)
{
    for (int k = 0; k < 8; ++k) {
        const int x = (home + k) & 7;
        const int lo = x * chunk;
        const int n = (nblk - lo < chunk) ? nblk - lo : chunk;
        if (n <= 0) continue;
        const uint32_t i = __hip_atomic_fetch_add(&ctr[x], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (i < (uint32_t)n) return lo + (int)i;
    }
    return -1;
}

// WM x WN wavefronts, each owning TM x TN MFMA tiles of 32 x 32.
template <int MODE, int WM, int WN, int TM, int TN>
__global__ __launch_bounds__(WM * WN * 64) void grouped_gemm_bf16_kernel(const KArgs p)
{
    static_assert(MODE == 1 || TN == 2, "mode 0 pairs one gate tile with one up tile per wavefront");
    constexpr int THREADS = WM * WN * 64;
    constexpr int MT_GROUP = (MODE == 0) ? MT_GROUP0 : MT_GROUP1;
    constexpr int BM = WM * TM * 32;           // rows of A per workgroup
    constexpr int BN = WN * TN * 32;           // rows of B per workgroup
    constexpr int BN_OUT = (MODE == 0) ? BN / 2 : BN;
    constexpr int A_CH = BM * 8 / THREADS;     // 16-byte chunks each thread copies per slice
    constexpr int B_CH = BN * 8 / THREADS;
    // the two stages are separate arrays so that the compiler can tell a copy into one stage from
    // the fragment reads of the other (no wait for the copy before those reads)
    __shared__ u32x4_t lds_a0[BM * 8], lds_a1[BM * 8];
    __shared__ u32x4_t lds_b0[BN * 8], lds_b1[BN * 8];
    static_assert(BM == BN, "the epilogue stages its bands in the second A stage and the second B stage alike");

    // Persistent workgroups.  Workgroup ids are dealt round-robin to the 8 XCDs, so workgroup b runs
    // on XCD b % 8.  XCD x owns the contiguous range [x * chunk, (x + 1) * chunk) of logical tiles
    // (in the grouped order described at MT_GROUP0) and its workgroups claim the tiles of that range
    // one after the other from a counter: at any time the workgroups of one XCD therefore work on
    // neighbouring tiles, which share A rows and expert weights through that XCD's L2.  Tile numbers
    // are claimed three tiles ahead of their use (the descriptor and the row indices of a tile are
    // each fetched a tile ahead).
    __shared__ int lds_claim[4];
    const int ntn = (p.n_out + BN_OUT - 1) / BN_OUT;
    const int n_mt = p.tile_expert ? *p.n_tiles : (p.dense_rows + BM - 1) / BM;
    const int nblk = n_mt * ntn;
    const int chunk = (nblk + 7) >> 3;
    const int home = blockIdx.x & 7;
    const int tid = threadIdx.x;
    if (tid == 0) {
        for (int j = 0; j < 3; ++j) lds_claim[j] = claim_tile(p.tile_ctr, home, chunk, nblk);
    }
    __syncthreads();
    const int q0 = lds_claim[0];
    int q_nx = lds_claim[1], q_nn = lds_claim[2];      // the next tile and the one after it (-1: none)
    if (q0 < 0) return;

    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int li = lane & 31, lh = lane >> 5;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);   // the same value, known to be wave-uniform

    // Direct-to-LDS copies: one instruction moves 64 lanes x 16 bytes into 1 KB of contiguous LDS
    // (lane l lands at base + 16 l), i.e. into 8 row slots x 8 chunk positions.  Each lane therefore
    // inverts the swizzle of ITS landing slot to find which (row, chunk) of the tile to fetch.
    // Wavefront w issues the copies of row-slot groups w, w + NWAVES, ...  Offsets are 32-bit byte
    // offsets from wave-uniform bases: gathered rows index all of A (the launcher checks that A
    // spans less than 4 GiB), contiguous rows are relative to the tile's first row, and B offsets
    // stay inside one expert matrix.
    constexpr int NWAVES = WM * WN;
    constexpr int COPIES = A_CH + B_CH;   // copy instructions per wavefront and slice
    static_assert((BN / 2) % (NWAVES * 8) == 0, "a copy instruction never straddles the gate and up halves of the B tile");
    const int land_rs = lane >> 3, land_cp = lane & 7;   // landing row slot (within the group), chunk position
    const int nk = p.k_dim / GM_BK;   // >= 1

    // ---- state of the tile being computed
    int expert, row0, rows, nt;
    uint32_t a_off[A_CH], b_off[B_CH];
    int a_row[A_CH];
    const char *a_base, *b_base0, *b_base1;
    floatx16_t zero16;
#pragma unroll
    for (int r = 0; r < 16; ++r) zero16[r] = 0.f;

    // (the tile list holds rows already limited to the tile height, so nothing here consumes a loaded
    // value: the loads are waited for where the descriptor is first used, a tile later)
#define GM_TILE_INFO(qq, E, R0, RS, NT)                                                             \
    {                                                                                               \
        const int logical_ = __builtin_amdgcn_readfirstlane(qq);                                    \
        const int blk_ = logical_ / (MT_GROUP * ntn), r_ = logical_ - blk_ * (MT_GROUP * ntn);      \
        int mt_ = blk_ * MT_GROUP;                                                                  \
        if (mt_ + MT_GROUP <= n_mt) {  /* a full group of row tiles: row tile fastest inside it */   \
            NT = r_ / MT_GROUP;                                                                     \
            mt_ += r_ - NT * MT_GROUP;                                                              \
        } else {                       /* the last, partial group */                                \
            const int left_ = n_mt - mt_;                                                           \
            NT = r_ / left_;                                                                        \
            mt_ += r_ - NT * left_;                                                                 \
        }                                                                                           \
        if (p.tile_expert) {                                                                        \
            E = list_entry(p.tile_expert, mt_);                                                     \
            R0 = list_entry(p.tile_row0, mt_);                                                      \
            RS = list_entry(p.tile_rows, mt_);                                                      \
        } else {                                                                                    \
            E = 0;                                                                                  \
            R0 = mt_ * BM;                                                                          \
            RS = p.dense_rows - R0;                                                                 \
            if (RS > BM) RS = BM;                                                                   \
        }                                                                                           \
    }
    // rows of A this thread copies (through slot -> token when gathered) for the tile at first slot R0
    // with RS valid rows; fetched a tile ahead, used by GM_TILE_OFFSETS
#define GM_TILE_ROWS(R0, RS, OUT)                                                                   \
    _Pragma("unroll") for (int i = 0; i < A_CH; ++i) {                                               \
        const int rs_ = (wave + NWAVES * i) * 8 + land_rs;                                          \
        const int r_ = rs_ ^ ((rs_ >> 3) & 1);                                                      \
        const int rr_ = r_ < (RS) ? r_ : (RS) - 1;                                                  \
        OUT[i] = p.row_gather ? p.row_gather[(R0) + rr_] : rr_;                                     \
    }
#define GM_TILE_OFFSETS()                                                                           \
    a_base = reinterpret_cast<const char *>(p.row_gather ? p.a : p.a + (int64_t)row0 * p.lda);      \
    b_base0 = reinterpret_cast<const char *>(p.b0 + (int64_t)expert * p.n_out * p.k_dim);           \
    b_base1 = (MODE == 0) ? reinterpret_cast<const char *>(p.b1 + (int64_t)expert * p.n_out * p.k_dim) \
                          : b_base0;                                                                \
    _Pragma("unroll") for (int i = 0; i < A_CH; ++i) {                                               \
        const int rs_ = (wave + NWAVES * i) * 8 + land_rs;                                          \
        const int r_ = rs_ ^ ((rs_ >> 3) & 1);                                                      \
        const int c_ = land_cp ^ (r_ & 7);                                                          \
        a_off[i] = (uint32_t)(((int64_t)a_row[i] * p.lda + c_ * 8) * 2);                                     \
    }                                                                                               \
    _Pragma("unroll") for (int i = 0; i < B_CH; ++i) {                                               \
        const int rs_ = (wave + NWAVES * i) * 8 + land_rs;                                          \
        const int r_ = rs_ ^ ((rs_ >> 3) & 1);                                                      \
        const int c_ = land_cp ^ (r_ & 7);                                                          \
        int brow_ = (MODE == 0) ? nt * (BN / 2) + (r_ & (BN / 2 - 1)) : nt * BN + r_;               \
        if (brow_ >= p.n_out) brow_ = p.n_out - 1;   /* ragged last n-tile: loads stay in bounds, stores are masked */ \
        b_off[i] = (uint32_t)(((int64_t)brow_ * p.k_dim + c_ * 8) * 2);                             \
    }
    // mode 0: row-slot groups below BN/2 rows hold gate rows, the others up rows (a group never straddles)
#define GM_COPY_SLICE(la, lb, k0)                                                                   \
    {                                                                                               \
        const char *ab_ = a_base + (k0) * 2;                                                        \
        const char *bb0_ = b_base0 + (k0) * 2;                                                      \
        const char *bb1_ = b_base1 + (k0) * 2;                                                      \
        _Pragma("unroll") for (int i = 0; i < A_CH; ++i)                                             \
            copy16_to_lds(ab_, a_off[i], &la[(wave_u + NWAVES * i) * 64]);                          \
        _Pragma("unroll") for (int i = 0; i < B_CH; ++i)                                             \
            copy16_to_lds((MODE == 0 && NWAVES * i * 8 >= BN / 2) ? bb1_ : bb0_, b_off[i],          \
                          &lb[(wave_u + NWAVES * i) * 64]);   /* whole groups: gate rows first, then up rows */ \
    }                                                                                               \
    __builtin_amdgcn_sched_barrier(0);   /* keep the copies where they are written */

    // fragment of k-step ks: row (tile base) + li, logical chunk 2 * ks + lh
    int fr_idx[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) fr_idx[ks] = lds_slot(li, 2 * ks + lh);
    const int a_tile0 = wm * TM * 32 * 8;                                       // + mi * 256
    const int b_tile0 = (MODE == 0) ? wn * 32 * 8 : wn * TN * 32 * 8;            // + ni * B_TILE_STEP
    constexpr int B_TILE_STEP = (MODE == 0) ? (BN / 2) * 8 : 32 * 8;

    // The j-th fragment read of a k-step, in the order in which the MFMAs (row tile slowest) first need
    // them: B 0, A 0, the other B fragments, the other A fragments.  All eight wavefronts ask the LDS
    // for their fragments at the same moment behind a barrier; the first MFMA can go once two reads
    // are back, not five.
#define GM_READ_ONE(la, lb, ks, fa, fb, j)                                                          \
    if ((j) == 0) fb[0] = *reinterpret_cast<const bf16x8_t *>(&lb[b_tile0 + fr_idx[ks]]);           \
    else if ((j) == 1) fa[0] = *reinterpret_cast<const bf16x8_t *>(&la[a_tile0 + fr_idx[ks]]);      \
    else if ((j) < 1 + TN) fb[((j) < 1 + TN && (j) >= 2) ? (j) - 1 : 0] =                           \
        *reinterpret_cast<const bf16x8_t *>(&lb[b_tile0 + fr_idx[ks] + ((j) - 1) * B_TILE_STEP]);   \
    else fa[((j) >= 1 + TN) ? (j) - TN : 0] =                                                       \
        *reinterpret_cast<const bf16x8_t *>(&la[a_tile0 + fr_idx[ks] + ((j) - TN) * 256]);
#define GM_READ_FRAGS(la, lb, ks, fa, fb)                                                           \
    _Pragma("unroll") for (int j_ = 0; j_ < TM + TN; ++j_) { GM_READ_ONE(la, lb, ks, fa, fb, j_) }
#define GM_MFMA(fa, fb)                                                                             \
    _Pragma("unroll") for (int mi = 0; mi < TM; ++mi)                                                \
        _Pragma("unroll") for (int ni = 0; ni < TN; ++ni)                                            \
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[ni], fa[mi], acc[mi][ni], 0, 0, 0);
    // the MFMAs of a k-step with the fragment reads of the next k-step dealt out behind the first of them
    // (issued in one block behind the barrier they would stand in the LDS queue in front of the other
    // wavefronts' first fragments); ZERO: start the accumulators from the constant zero
    // Only the first FRONT reads of the k-step's own fragments go out in front of its MFMAs (what the
    // first two MFMAs need); the rest follow behind the first MFMAs, then the next k-step's.
    constexpr int FRONT = 1 + TN;
    static_assert(TM * TN >= FRONT - 1 + TM + TN, "a k-step has enough MFMAs to deal the reads out behind");
#define GM_MFMA_READS(fa, fb, ZERO, la, lb, ks, fa_nx, fb_nx)                                       \
    _Pragma("unroll") for (int mi = 0; mi < TM; ++mi)                                                \
        _Pragma("unroll") for (int ni = 0; ni < TN; ++ni) {                                          \
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[ni], fa[mi], (ZERO) ? zero16 : acc[mi][ni], 0, 0, 0); \
            __builtin_amdgcn_sched_barrier(0);                                                      \
            if (mi * TN + ni < TM + TN - FRONT) { GM_READ_ONE(la, lb, (ks) - 1, fa, fb, FRONT + mi * TN + ni) } \
            if (mi * TN + ni >= FRONT - 1 && mi * TN + ni < FRONT - 1 + TM + TN) {                  \
                GM_READ_ONE(la, lb, ks, fa_nx, fb_nx, mi * TN + ni - (FRONT - 1))                   \
            }                                                                                       \
            __builtin_amdgcn_sched_barrier(0);                                                      \
        }
    // the same with the reads of two k-steps, two reads behind each of the first MFMAs (all of them are
    // then on their way two MFMAs before the barrier that waits for them)
#define GM_MFMA_READS2(fa, fb, la, lb, ks_a, fa_a, fb_a, ks_b, fa_b, fb_b)                          \
    _Pragma("unroll") for (int mi = 0; mi < TM; ++mi)                                                \
        _Pragma("unroll") for (int ni = 0; ni < TN; ++ni) {                                          \
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[ni], fa[mi], acc[mi][ni], 0, 0, 0); \
            __builtin_amdgcn_sched_barrier(0);                                                      \
            if (mi * TN + ni < TM + TN) { GM_READ_ONE(la, lb, ks_a, fa_a, fb_a, mi * TN + ni) }     \
            if (mi * TN + ni < TM + TN) { GM_READ_ONE(la, lb, ks_b, fa_b, fb_b, mi * TN + ni) }     \
            __builtin_amdgcn_sched_barrier(0);                                                      \
        }
    // copy instruction c of a slice (0 .. A_CH-1: A rows, then B rows)
#define GM_COPY_ONE(la, lb, k0, c)                                                                  \
    if ((c) < A_CH)                                                                                 \
        copy16_to_lds(a_base + (k0) * 2, a_off[(c) < A_CH ? (c) : 0], &la[(wave_u + NWAVES * (c)) * 64]); \
    else                                                                                            \
        copy16_to_lds(((MODE == 0 && NWAVES * ((c) - A_CH) * 8 >= BN / 2) ? b_base1 : b_base0) + (k0) * 2, \
                      b_off[(c) >= A_CH ? (c) - A_CH : 0], &lb[(wave_u + NWAVES * ((c) - A_CH)) * 64]);
    // the MFMAs of one k-step with copy instructions of a slice dealt out between them, one behind
    // every COPY_EVERY-th MFMA starting with copy c0, so that the wavefront never queues several
    // copies at once (a full address queue stalls the wavefront, MFMAs included).  The compute
    // unit's memory path takes a slice's 64 copies of 1 KB at 64 bytes per cycle, as long as the
    // MFMAs of two k-steps: the copies are therefore spread over the last two k-steps of a slice.
    constexpr int COPY_EVERY = 2;
    static_assert(COPIES * COPY_EVERY == 2 * TM * TN, "a slice's copies are dealt out over the MFMAs of two k-steps");
#define GM_MFMA_COPIES(fa, fb, la, lb, k0, on, c0)                                                  \
    _Pragma("unroll") for (int mi = 0; mi < TM; ++mi)                                                \
        _Pragma("unroll") for (int ni = 0; ni < TN; ++ni) {                                          \
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[ni], fa[mi], acc[mi][ni], 0, 0, 0); \
            __builtin_amdgcn_sched_barrier(0);                                                      \
            if ((mi * TN + ni) % COPY_EVERY == 0 && (on)) { GM_COPY_ONE(la, lb, k0, (c0) + (mi * TN + ni) / COPY_EVERY) } \
            __builtin_amdgcn_sched_barrier(0);                                                      \
        }
    // k-steps of one slice, three fragment buffers: the fragments of step 1 are read under the MFMAs of
    // step 0, those of steps 2 and 3 under the MFMAs of step 1 (step 3 into the buffer step 0 has
    // left).  MID runs behind the MFMAs of step 1, when every fragment of the stage has been requested
    // a while ago: it waits for the last of them, passes a barrier and may then refill the stage, two
    // k-steps before the slice ends, so a copy has a slice and a half of MFMA time to land.
#define GM_COMPUTE(la, lb, STEP0, MID, LAST)                                                            \
    {                                                                                               \
        bf16x8_t fa0[TM], fb0[TN], fa1[TM], fb1[TN], fa2[TM], fb2[TN];                              \
        _Pragma("unroll") for (int j_ = 0; j_ < FRONT; ++j_) { GM_READ_ONE(la, lb, 0, fa0, fb0, j_) } \
        __builtin_amdgcn_sched_barrier(0);                                                          \
        STEP0(fa0, fb0, la, lb, fa1, fb1)                                                           \
        __builtin_amdgcn_sched_barrier(0);                                                          \
        GM_MFMA_READS2(fa1, fb1, la, lb, 2, fa2, fb2, 3, fa0, fb0)                                  \
        __builtin_amdgcn_sched_barrier(0);                                                          \
        MID                                                                                         \
        __builtin_amdgcn_sched_barrier(0);                                                          \
        LAST(fa2, fb2, 0)                                                                           \
        __builtin_amdgcn_sched_barrier(0);                                                          \
        LAST(fa0, fb0, TM * TN / COPY_EVERY)                                                        \
    }
    // Workgroup barrier that orders LDS traffic only.  (__syncthreads would also wait for every
    // direct-to-LDS copy in flight.)
#define GM_LDS_BARRIER() asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory")
    // this wavefront's copies of one slice have landed once at most `later` younger vector memory
    // operations are outstanding (they complete in order); then everyone's have
    static_assert(COPIES == 8, "the wait immediates below are written for 8 copies per slice");
#define GM_WAIT_SLICE(more_in_flight)                                                               \
    if (more_in_flight) __builtin_amdgcn_s_waitcnt(0x0F78); /* vmcnt(8) */                          \
    else __builtin_amdgcn_s_waitcnt(0x0F70);                /* vmcnt(0) */                          \
    GM_LDS_BARRIER();

    // Epilogue of one 32-row band per wavefront row (mi).  The MFMAs take the B rows as their first
    // operand, so an accumulator holds the transposed 32 x 32 tile: a lane owns ONE row of A (li) and,
    // per group of four registers g, the four adjacent output columns 8 g + 4 lh + (0..3).  Four
    // registers therefore pack into 8 contiguous bytes of one output row.  Each band of the workgroup
    // tile (both wm halves, all
    // BN_OUT columns) is staged in LDS as bf16 and written out as 16-byte chunks, so every output row
    // leaves as one contiguous run of full cache lines.  The 16-byte chunk c of band row R is stored
    // at chunk position c ^ (R & 7): the eight rows li..li+7 that write the same logical chunk then
    // fall on different banks.  Bands 0 and 2 are staged in the second A stage,
    // bands 1 and 3 in the second B stage (both idle after the last slice), two bands per barrier,
    // and the first stage is free to receive the next tile's first slice meanwhile.
    constexpr int ROWB = BN_OUT * 2;        // bytes per staged row
    constexpr int CPR = BN_OUT / 8;         // 16-byte chunks per staged row
    static_assert(CPR % 8 == 0, "the chunk swizzle permutes groups of eight chunks");
    // accumulators of band mi -> staging array st (u32x4_t[], indexed in bytes)
#define GM_EPI_STAGE(mi, st)                                                                        \
    {                                                                                               \
        char *reg = reinterpret_cast<char *>(st) + (wm * 32 + li) * ROWB + lh * 8;                  \
        _Pragma("unroll") for (int ni = 0; ni < ((MODE == 0) ? 1 : TN); ++ni) {                      \
            const int seg = (MODE == 0) ? wn : wn * TN + ni;                                        \
            _Pragma("unroll") for (int g = 0; g < 4; ++g) {                                          \
                float v[4];                                                                         \
                _Pragma("unroll") for (int e = 0; e < 4; ++e) {                                      \
                    if (MODE == 0) {                                                                \
                        const float gt = acc[mi][0][4 * g + e], up = acc[mi][1][4 * g + e];         \
                        v[e] = gt * up * __builtin_amdgcn_rcpf(1.0f + __expf(-gt));   /* silu(g) * u; the 1-ulp reciprocal is far inside bf16 rounding */ \
                    } else {                                                                        \
                        v[e] = acc[mi][ni][4 * g + e];                                              \
                    }                                                                               \
                }                                                                                   \
                u32x2_t pk;                                                                         \
                pk.x = pack_bf16x2(v[0], v[1]);                                                     \
                pk.y = pack_bf16x2(v[2], v[3]);                                                     \
                *reinterpret_cast<u32x2_t *>(reg + (((seg * 4 + g) ^ (li & 7)) << 4)) = pk;         \
            }                                                                                       \
        }                                                                                           \
    }
    // staging array st -> global memory, 16 bytes per lane (non-temporal: the output is not read again by
    // this kernel and should not push operand lines out of the L2; the last band of the down projection
    // is stored the ordinary way, which is acknowledged sooner: the next tile's first wait on the vector
    // memory counter also waits for these stores).  e_base is the wave-uniform address
    // of the tile's first output element; offsets inside a tile fit 32 bits (checked by the launcher).
#define GM_EPI_STORE2(mi_a, st_a, mi_b, st_b, e_base, e_rows, e_cols)                               \
    {                                                                                               \
        constexpr int NJ = 64 * CPR / THREADS;                                                      \
        const int R0 = tid / CPR, ch = tid % CPR;   /* band row over both wm halves, chunk in the row */ \
        u32x4_t v[2][NJ];                                                                           \
        _Pragma("unroll") for (int j = 0; j < NJ; ++j) {                                             \
            const int R = R0 + j * (THREADS / CPR);                                                 \
            v[0][j] = *reinterpret_cast<const u32x4_t *>(reinterpret_cast<const char *>(st_a) + R * ROWB + ((ch ^ (R & 7)) << 4)); \
            v[1][j] = *reinterpret_cast<const u32x4_t *>(reinterpret_cast<const char *>(st_b) + R * ROWB + ((ch ^ (R & 7)) << 4)); \
        }                                                                                           \
        static_assert(NJ == 2 || NJ == 4, "the pin below is written for two or four chunks per thread"); \
        /* Every LDS read of both bands is issued before the first store (a read would otherwise sink  \
           into its store's branch, behind stores that can stand in a full queue).  The staging areas   \
           are the landing zone of the next tile's second slice, whose copies a wavefront issues once   \
           its own stores are out: by then every other wavefront's reads, a dozen instructions behind   \
           the barrier, are long done, and the copied data is an L2 round trip further away. */         \
        if (NJ == 4) asm volatile("" : "+v"(v[0][0]), "+v"(v[0][1]), "+v"(v[0][NJ - 2]), "+v"(v[0][NJ - 1]), \
                                       "+v"(v[1][0]), "+v"(v[1][1]), "+v"(v[1][NJ - 2]), "+v"(v[1][NJ - 1])); \
        else asm volatile("" : "+v"(v[0][0]), "+v"(v[0][1]), "+v"(v[1][0]), "+v"(v[1][1]));         \
        _Pragma("unroll") for (int b = 0; b < 2; ++b)                                                \
            _Pragma("unroll") for (int j = 0; j < NJ; ++j) {                                         \
                const int mi_ = b ? (mi_b) : (mi_a);                                                \
                const int R = R0 + j * (THREADS / CPR);                                             \
                const int m = ((R >> 5) * TM + mi_) * 32 + (R & 31);                                \
                if (m < (e_rows) && ch * 8 < (e_cols)) {                                            \
                    u32x4_t *dst_ = reinterpret_cast<u32x4_t *>((e_base) + ((uint32_t)m * ldc_bytes + (uint32_t)ch * 16u)); \
                    if (MODE == 1 && mi_ == TM - 1) *dst_ = v[b][j];                                \
                    else __builtin_nontemporal_store(v[b][j], dst_);                                \
                }                                                                                   \
            }                                                                                       \
    }

    GM_TILE_INFO(q0, expert, row0, rows, nt)
    GM_TILE_ROWS(row0, rows, a_row)
    GM_TILE_OFFSETS()
    GM_COPY_SLICE(lds_a0, lds_b0, 0)
    // descriptor of this workgroup's next tile
    bool has_next = q_nx >= 0;
    int nx_expert = 0, nx_row0 = 0, nx_rows = 1, nx_nt = 0;
    if (has_next) GM_TILE_INFO(q_nx, nx_expert, nx_row0, nx_rows, nx_nt)

    uint32_t claim_raw = 0;      // ticket of the claim in flight (lane 0 only; read only when one was made)
    for (;;) {
        // Fetched under the main loop: the next tile's row indices (its descriptor
        // arrived a tile ago) and the descriptor of the tile after it.  The descriptor goes out now
        // (scalar loads); the vector loads and the claim go out behind the first wait below, so that
        // the wait for slice 0 is not also a wait for their round trip.
        int a_row_nx[A_CH];
        const bool has_nn = q_nn >= 0;
        int nn_expert = 0, nn_row0 = 0, nn_rows = 1, nn_nt = 0;
        if (has_nn) GM_TILE_INFO(q_nn, nn_expert, nn_row0, nn_rows, nn_nt)

        floatx16_t acc[TM][TN];   // first written by the MFMAs of slice 0, k-step 0

        // Main loop.  Slice 0 is already on its way into stage 0; even slices use stage 0, odd ones
        // stage 1.  A stage is refilled with the slice after next as soon as all its fragments have
        // been read (inside GM_COMPUTE), so a copy has about one and a half slices of MFMA time to land.
        if (nk > 1) { GM_COPY_SLICE(lds_a1, lds_b1, GM_BK) }
        GM_WAIT_SLICE(nk > 1)
        // the claim for the tile three ahead (this XCD's own counter) is looked at when the main loop
        // is over: nobody waits for the atomic's round trip
        // (the counter's address is handed over in a vector register: for an atomic with a wave-uniform
        // address the compiler emits a wave-wide reduction that waits for the result on the spot)
        if (threadIdx.x == 0 && has_nn) {
            typedef uint32_t __attribute__((address_space(1))) *global_u32_ptr;
            uintptr_t ctr_addr = reinterpret_cast<uintptr_t>(p.tile_ctr + home);
            asm volatile("" : "+v"(ctr_addr));
            claim_raw = __hip_atomic_fetch_add((global_u32_ptr)ctr_addr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        {
            int tid_early = threadIdx.x;
            asm volatile("" : "+v"(tid_early));   // (index arithmetic redone here rather than kept in registers)
            const int tid = tid_early;
            const int lane = tid & 63, wave = tid >> 6;
            const int land_rs = lane >> 3;
            if (has_next) {
                GM_TILE_ROWS(nx_row0, nx_rows, a_row_nx)
            } else {
#pragma unroll
                for (int i = 0; i < A_CH; ++i) a_row_nx[i] = 0;
            }
        }
#define GM_STEP0_EVEN(fa, fb, la, lb, fa_nx, fb_nx)                                                 \
    if (kt == 0) { GM_MFMA_READS(fa, fb, 1, la, lb, 1, fa_nx, fb_nx) } else { GM_MFMA_READS(fa, fb, 0, la, lb, 1, fa_nx, fb_nx) }
#define GM_STEP0_ODD(fa, fb, la, lb, fa_nx, fb_nx) GM_MFMA_READS(fa, fb, 0, la, lb, 1, fa_nx, fb_nx)
#define GM_LAST_REFILL0(fa, fb, c0) GM_MFMA_COPIES(fa, fb, lds_a0, lds_b0, (kt + 2) * GM_BK, refill0, c0)
#define GM_LAST_REFILL1(fa, fb, c0) GM_MFMA_COPIES(fa, fb, lds_a1, lds_b1, (kt + 3) * GM_BK, refill1, c0)
        for (int kt = 0; kt < nk; kt += 2) {
            const bool refill0 = kt + 2 < nk;
            GM_COMPUTE(lds_a0, lds_b0, GM_STEP0_EVEN, GM_LDS_BARRIER();, GM_LAST_REFILL0)
            if (kt + 1 < nk) {
                const bool refill1 = kt + 3 < nk;
                GM_WAIT_SLICE(refill0)
                GM_COMPUTE(lds_a1, lds_b1, GM_STEP0_ODD, GM_LDS_BARRIER();, GM_LAST_REFILL1)
                if (refill0) { GM_WAIT_SLICE(refill1) }
            }
        }

        // Every copy has landed; the loads and the claim issued under the loop have too.  Saying so on
        // every path keeps the compiler from waiting for them again at the top of the next tile, where
        // the wait would be for this tile's stores.
        __builtin_amdgcn_s_waitcnt(0x0F70);   /* vmcnt(0) */
        // the claim made at the top of this tile: inside this XCD's range, or else one from another's
        if (threadIdx.x == 0) {
            int q3 = -1;
            if (has_nn) {
                const int lo = home * chunk;
                const int n_home = (nblk - lo < chunk) ? nblk - lo : chunk;
                q3 = (claim_raw < (uint32_t)(n_home > 0 ? n_home : 0)) ? lo + (int)claim_raw
                                                                        : claim_tile(p.tile_ctr, home, chunk, nblk);
            }
            lds_claim[3] = q3;
        }
        // Both stages are idle now.  The finished tile is written out band by band while the next
        // tile's row indices, offsets and first slice are fetched in between.
        // (Thread-index arithmetic of this phase is redone per tile from a value the optimiser
        // cannot see through, so that none of it is hoisted and kept in registers across the main loop.)
        int tid_again = threadIdx.x;
        asm volatile("" : "+v"(tid_again));
        const int tid = tid_again;
        const int lane = tid & 63, wave = tid >> 6;
        const int wm = wave / WN, wn = wave % WN;
        const int li = lane & 31, lh = lane >> 5;
        const int land_rs = lane >> 3, land_cp = lane & 7;
        const int wave_u = __builtin_amdgcn_readfirstlane(wave);
        const int e_rows = rows;
        const int e_cols = p.n_out - nt * BN_OUT;      // valid columns of this n-tile (the store masks the rest)
        char *const e_base = reinterpret_cast<char *>(p.c + (p.c_row_offset + row0) * p.ldc + nt * BN_OUT);
        const uint32_t ldc_bytes = (uint32_t)p.ldc * 2u;
        if (has_next) {
            expert = nx_expert; row0 = nx_row0; rows = nx_rows; nt = nx_nt;
#pragma unroll
            for (int i = 0; i < A_CH; ++i) a_row[i] = a_row_nx[i];
        }
        static_assert(TM == 4, "the epilogue is written out for four bands");
        GM_EPI_STAGE(0, lds_a1)
        if (has_next) {
            GM_TILE_OFFSETS()
            GM_COPY_SLICE(lds_a0, lds_b0, 0)
        }
        GM_EPI_STAGE(1, lds_b1)
        GM_LDS_BARRIER();
        GM_EPI_STORE2(0, lds_a1, 1, lds_b1, e_base, e_rows, e_cols)
        GM_LDS_BARRIER();      // everyone has read bands 0 and 1
        GM_EPI_STAGE(2, lds_a1)
        GM_EPI_STAGE(3, lds_b1)
        GM_LDS_BARRIER();
        GM_EPI_STORE2(2, lds_a1, 3, lds_b1, e_base, e_rows, e_cols)
        if (!has_next) break;
        has_next = has_nn;
        nx_expert = nn_expert; nx_row0 = nn_row0; nx_rows = nn_rows; nx_nt = nn_nt;
        q_nn = lds_claim[3];       // written before the epilogue's barriers
    }
}

// tile configuration in use: 2 x 4 wavefronts of 4 x 2 MFMA tiles = 256 x 256
constexpr int CFG_WM = 2, CFG_WN = 4, CFG_TM = 4, CFG_TN = 2;
constexpr int CFG_BM = CFG_WM * CFG_TM * 32;
constexpr int CFG_BN = CFG_WN * CFG_TN * 32;

}  // namespace

int gemm_tile_m() { return CFG_BM; }

remoe_status launch_grouped_gemm_bf16(int mode, const GroupedGemmArgs &g, hipStream_t stream)
{
    const int bn = (mode == 0) ? CFG_BN / 2 : CFG_BN;
    if (g.k_dim % GM_BK != 0 || g.n_out < 1)
        return fail(REMOE_E_UNSUPPORTED, "bf16 GEMM needs k %% 64 == 0 (k=%d n=%d)", g.k_dim, g.n_out);
    if (g.row_gather && g.a_rows * g.lda * 2 >= (int64_t)1 << 32)
        return fail(REMOE_E_UNSUPPORTED, "gathered GEMM operand spans 4 GiB or more (%lld rows)", (long long)g.a_rows);
    if ((int64_t)g.n_out * g.k_dim * 2 >= (int64_t)1 << 32)
        return fail(REMOE_E_UNSUPPORTED, "one expert matrix spans 4 GiB or more");
    if (g.ldc * 2 * CFG_BM >= (int64_t)1 << 32 || g.n_out % 8 != 0)
        return fail(REMOE_E_UNSUPPORTED, "bf16 GEMM output needs n %% 8 == 0 and a row pitch below 8 Mi elements (n=%d ldc=%lld)",
                    g.n_out, (long long)g.ldc);
    if (g.row_scale) return fail(REMOE_E_INVALID_ARG, "the bf16 GEMM applies no row factors (the combine step does)");
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
    p.c = static_cast<bf16_t *>(g.c);
    p.ldc = g.ldc;
    p.c_row_offset = g.c_row_offset;
    p.tile_ctr = g.tile_ctr;
    if (!p.tile_ctr) return fail(REMOE_E_INVALID_ARG, "grouped_gemm_bf16 needs tile counters");
    // persistent launch: one workgroup per compute unit (a multiple of 8, one share per XCD), fewer
    // when the upper bound of tiles is smaller
    int dev = 0, n_cu = 0;
    REMOE_HIP_TRY(hipGetDevice(&dev));
    REMOE_HIP_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
    const int64_t nblk = (int64_t)g.max_tiles * ceil_div(g.n_out, bn);
    int64_t n_wg = ceil_div(nblk, 8) * 8;
    const int64_t resident = n_cu >= 8 ? (int64_t)(n_cu / 8) * 8 : 8;
    if (n_wg > resident) n_wg = resident;
    const dim3 grid((unsigned)n_wg), block(CFG_WM * CFG_WN * 64);
    if (mode == 0)
        hipLaunchKernelGGL((grouped_gemm_bf16_kernel<0, CFG_WM, CFG_WN, CFG_TM, CFG_TN>), grid, block, 0, stream, p);
    else
        hipLaunchKernelGGL((grouped_gemm_bf16_kernel<1, CFG_WM, CFG_WN, CFG_TM, CFG_TN>), grid, block, 0, stream, p);
    return check_hip(hipGetLastError(), "grouped_gemm_bf16 launch");
}

}  // namespace remoe
