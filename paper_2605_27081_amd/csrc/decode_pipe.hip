// M = 1 decode with the layers of a step overlapped: one layer per XCD at a time, software pipeline
// over each XCD's layers.
//
// Per layer-step the work is the same as in the layer-chained kernel: the fp32 router matrix and the
// three matrices of the K selected experts are streamed once from HBM (Sec. 3.1 routing; the B = 1
// regime of Sec. 3), about one flop per byte.  What differs is who works on what, and when.  Every
// layer of a step reads the same input row, so the layers of one step do not depend on each other:
//
//   * The workgroups are split into 8 groups (workgroup b belongs to group b % 8: with round-robin
//     dispatch that is one XCD per group).  Group x owns layers x, x + 8, x + 16, ...  A layer-step is
//     therefore spread over 32 compute units instead of 256: eight times more bytes per exchange
//     between workgroups, so the fixed cost of those exchanges is amortised eight times better.
//   * Inside a group the two exchanges a layer needs (all partial logits before the top-k, all SwiGLU
//     activations before the down projection) are each given a pipeline stage to arrive instead of a
//     barrier.  Iteration i of a step works on the group's layers number
//         R(i)    partial router logits                                   -> published, tagged
//         T(i-1)  top-k / softmax from the logits published an iteration ago (one wavefront per
//                 workgroup, in turn; the result is first used at the end of the iteration)
//         G(i-2)  gate/up rows of the selected experts, SwiGLU            -> published, tagged
//         D(i-4)  down projection from the activations published two iterations ago
//     in the order R, T, G, D.  G's activations are split statically over the wavefronts of the
//     group; D's output rows are split statically over the workgroups and handed out one at a time
//     inside a workgroup (an LDS counter), so its wavefronts reach the next barrier together
//     however unevenly memory served them.
//
// Exchanged values carry the number of the layer-step that produced them (partial logits: fp32 and a
// 32-bit tag; three SwiGLU activations of one wavefront: 3 x bf16 and a 16-bit tag, one 8-byte word),
// so a reader needs no barrier: it polls (agent-scope loads, which bypass the per-XCD L2 and its stale
// copies) until the tags match, and in steady state they already do; a missing word is asked for
// again by the wavefront that needs it.  Everything an iteration needs at its start is requested from
// inside the previous one (the polls before its down projection, the router segments and the first
// gate / up rows behind it), so HBM keeps streaming across iterations.  The streaming loops are
// branch-free with a fixed number of loads per unit of work: the compiler's wait counts then let one
// register set be reduced while the other's loads stay in flight.  Weight pointers come out of the
// launch's table through scalar loads (a vector load would sit in the same in-order queue as the
// weight stream).  bf16 activations are what the batched path stores between its two GEMMs as well;
// they let the gate/up and the down products run as packed bf16 dot instructions (exact products,
// fp32 accumulation) against x and h kept in bf16 in LDS.  Steps stay strictly sequential: a grid
// barrier over all workgroups closes every step (the statistics of step t+1 need those of step t, and
// a decoder would need the step's output before it has the next input).
//
// One workgroup of 8 wavefronts per compute unit; every wait is bounded as in the chained kernel.
#include "common.h"
#include "decode_common.h"
#include "topk.h"

namespace remoe {

namespace {

constexpr int DP_THREADS = DEC_THREADS;
constexpr int DP_WAVES = DP_THREADS / 64;
constexpr int DP_GROUPS = DEC_GROUPS; // groups of workgroups, each on its own layers (one per XCD)
constexpr int DP_MAX_KI = 6144;      // K * I activations of one layer
constexpr int DP_MAX_DCH = 12;       // down-projection 16-byte chunks per lane per output row
constexpr int DP_POLL_L = 4;         // tagged logit words per thread (N * H / 256 <= 2048)
constexpr int DP_POLL_H = 4;         // activation words per thread (<= 2048 words per layer)
constexpr int DP_MAX_R = 4;          // router segments per wavefront, fetched ahead
constexpr int DP_SEL = 8;            // layers whose selection is kept (a layer's is used for 4 iterations)

struct PipeArgs {
    const void *const *layers;   // [L][4] device pointers: w_router, w_gate, w_up, w_down
    const bf16_t *x;             // [T_total, H]
    int64_t steps_total, step0, n_steps;
    int n_layers, H, N, I, K, renorm;
    bf16_t *y;                   // [T_total, L, H]
    int32_t *out_idx;            // [L, T_total, K]
    float *out_w;                // [L, T_total, K]
    int n_caps;
    int caps[DEC_MAX_CAPS];
    unsigned long long expert_bytes;
    uint32_t *lru_state;
    uint8_t *out_overlap;
    uint8_t *out_miss;
    unsigned long long *sum_overlap;
    unsigned long long *total_miss;
    unsigned long long *bytes_fetched;
    unsigned long long *logit_ring;   // [groups][DEC_RING][N * H / 256]  (tag << 32) | float bits
    unsigned long long *h_ring;       // [groups][DEC_RING][h_slot]: 3 x bf16 | tag16 << 48 per word
    int h_slot;                       // words per ring slot
    uint32_t *bar;
    uint32_t *abort_flag;
    unsigned long long spin_limit;
};

// Workgroup barrier that orders LDS traffic only (a full __syncthreads would also wait for every
// weight load in flight, which is exactly what must keep flying).
#define DP_LDS_BARRIER() asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory")

// 16-bit tag of a layer-step (never 0, the value of a cleared word).  A ring slot is rewritten every
// DEC_RING layers of its group, so a word 65535 layer-steps old cannot survive to be mistaken for a
// new one.
__device__ __forceinline__ uint32_t tag16(uint32_t tag) { return tag % 65535u + 1u; }

__device__ __forceinline__ unsigned long long poll_word(const unsigned long long *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// XCH: 16-byte chunks per lane of one hidden row (hidden / 512).  DCH: 16-byte chunks per lane of one
// down-projection output row over the K selected experts (K * inter / 512, rounded up to a supported
// count).  Both fix the number of loads per unit of work at compile time: the steady-state loops
// below then contain no branch, and the compiler can wait for exactly the loads an instruction needs
// while the next unit's loads stay in flight.
template <int XCH, int DCH>
__global__ __launch_bounds__(DP_THREADS) void decode_pipe_kernel(const PipeArgs a)
{
    __shared__ __attribute__((aligned(16))) bf16_t hl[2][DP_MAX_KI];   // activations of two layers (bf16)
    __shared__ __attribute__((aligned(16))) bf16_t xs[4096];           // the step's input row
    __shared__ float lpart[2][128 * 16]; // partial logits of the layer being ranked (two iterations apart)
    __shared__ int sel_e[DP_SEL][8];     // selections of the group's last DP_SEL layers: written by the wavefront
    __shared__ float sel_w[DP_SEL][8];   // on top-k duty, read by everyone from the next iteration on
    __shared__ uint32_t sel_tag[DP_SEL]; // tag of the layer-step whose selection a slot of sel_e / sel_w holds
    __shared__ uint32_t row_ctr[4];      // next output row of the workgroup's share, per iteration (mod 4)
    __shared__ int behind_lds;           // set when a wait ran out: the workgroup returns
    __shared__ int bar_ok;
    __shared__ TraceLds ts;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // known to be the same in every lane: what derives from it stays in scalar registers
    const int G = gridDim.x;
    const int NG = (G % DP_GROUPS == 0) ? DP_GROUPS : 1;   // groups
    const int group = blockIdx.x % NG;
    const int gr = blockIdx.x / NG;                      // this workgroup's rank in its group
    const int GS = G / NG;                               // workgroups per group
    const int W = GS * DP_WAVES;                         // wavefronts per group
    const int gw = gr * DP_WAVES + wave;                 // this wavefront's index in its group
    const int H = a.H, N = a.N, I = a.I, K = a.K, L = a.n_layers;
    const int segs = H / DEC_SEG;
    const int KI = K * I;
    const int n_items1 = N * segs;
    const int ipw = (KI + W - 1) / W;                    // activations per wavefront
    const int wpw = (ipw + 2) / 3;                       // exchange words per wavefront (3 activations each)
    const int n_words = W * wpw;                         // <= DP_POLL_H * DP_THREADS (checked by the launcher)
    const int rows_per_wg = (H + GS - 1) / GS;
    const int dchunks = KI / 8;
    const int chunks_per_row = I / 8;
    const int n_mine = group < L ? (L - group + NG - 1) / NG : 0;      // layers group, group + NG, ...
    const bool stats_wave = gr == GS - 1 && wave == DP_WAVES - 1;
    unsigned long long *const logit_ring = a.logit_ring + (size_t)group * DEC_RING * n_items1;
    unsigned long long *const h_ring = a.h_ring + (size_t)group * DEC_RING * a.h_slot;
    uint32_t bar_phase = 0;

    if (gr == GS - 1) {                                  // trace state of this group's layers -> LDS
        for (int q = tid; q < n_mine * 128; q += DP_THREADS) {
            const int l = group + NG * (q >> 7), e = q & 127;
            ts.last[l][e] = (e < N) ? a.lru_state[l * N + e] : 0u;
        }
        for (int q = tid; q < n_mine; q += DP_THREADS) {
            const int l = group + NG * q;
            ts.sum_ov[l] = a.sum_overlap[l];
            for (int c = 0; c < a.n_caps; ++c) ts.tot[c][l] = a.total_miss[c * L + l];
        }
    }
    if (tid == 0) behind_lds = 0;
    if (tid < DP_SEL) sel_tag[tid] = 0u;                 // tag 0 = no layer-step
    if (tid < 4) row_ctr[tid] = 0u;
    __syncthreads();

    // ---- per-wavefront constants ---------------------------------------------------------------------
    const int item0 = gw * ipw;
    int nit = KI - item0;
    if (nit > ipw) nit = ipw;
    if (nit < 0) nit = 0;
    const int wg_row0 = gr * rows_per_wg;                // this workgroup's share of a layer's output rows
    int wg_rows = H - wg_row0;
    if (wg_rows > rows_per_wg) wg_rows = rows_per_wg;
    if (wg_rows < 0) wg_rows = 0;
    // chunk q of a wavefront's down-row work is chunk q % chunks_per_row of expert slot q / chunks_per_row;
    // the quotient by multiplication (exact for q < 2^16, chunks_per_row <= 2^16)
    const uint32_t cpr_magic = (uint32_t)((0x100000000ull + (unsigned)chunks_per_row - 1) / (unsigned)chunks_per_row);
#define DP_SLOT_OF(q) ((int)__umulhi((uint32_t)(q), cpr_magic))
    const int loff = lane * 8;

#pragma unroll 1
    for (int64_t s = 0; s < a.n_steps; ++s) {
        const int64_t g = a.step0 + s;
        const bf16_t *xg = a.x + g * H;
        const uint32_t tag0 = (uint32_t)(g * L) + 1u;    // tag of layer l of this step: tag0 + l

        // x of this step lives in LDS as bf16 (registers are needed for loads in flight);
        // the previous step's last readers are behind the grid barrier that closed it
        for (int k = tid; k < H / 8; k += DP_THREADS)
            *reinterpret_cast<u32x4_t *>(&xs[k * 8]) = *reinterpret_cast<const u32x4_t *>(xg + k * 8);
        DP_LDS_BARRIER();

        // registers that carry loads across the iteration boundary
        unsigned long long pl[DP_POLL_L], ph[DP_POLL_H];
        u32x4_t dvA[DCH], dvB[DCH];
        u32x4_t gA[XCH], uA[XCH], gB[XCH], uB[XCH];
        floatx4_t wr[DP_MAX_R];

        // Output row `row` of layer number md_ (all K experts' pieces of it) -> dv.  A row number past
        // the workgroup's share (valid_ false) turns every load into one of the tensor's first bytes:
        // the number of loads per call stays fixed, which is what lets the loop below wait precisely.
#define DP_LOAD_DROW(dv, md_, row, valid_)                                                            \
    {                                                                                                 \
        int lane_ = threadIdx.x & 63;                                                                 \
        asm volatile("" : "+v"(lane_));   /* offsets are recomputed here, not kept in registers */     \
        const char *wd_ = static_cast<const char *>(table_ptr(a.layers, (group + NG * (md_)) * 4 + 3)); \
        const int *se_ = sel_e[(md_) & (DP_SEL - 1)];                                                 \
        _Pragma("unroll") for (int c = 0; c < DCH; ++c) {                                              \
            int q_ = c * 64 + lane_;                          /* past the end: the last chunk again, */ \
            if (q_ >= dchunks) q_ = dchunks - 1;              /* weighted 0 when the row is reduced  */ \
            const int j_ = DP_SLOT_OF(q_);                                                            \
            uint32_t off_ = (uint32_t)(((int64_t)se_[j_] * H + (row)) * I * 2) + (uint32_t)(q_ - j_ * chunks_per_row) * 16u; \
            if (!(valid_)) off_ = 0;                                                                  \
            dv[c] = load_global_stream<u32x4_t>(wd_ + off_);                                                 \
        }                                                                                             \
    }

        // gate and up rows of the next activation of layer number mg_ (expert slot g_j, index g_i)
#define DP_LOAD_ITEM(gv, uv, mg_)                                                                     \
    {                                                                                                 \
        const int e_ = __builtin_amdgcn_readfirstlane(sel_e[(mg_) & (DP_SEL - 1)][g_j]);              \
        const bf16_t *gp_ = static_cast<const bf16_t *>(table_ptr(a.layers, (group + NG * (mg_)) * 4 + 1)) + ((int64_t)e_ * I + g_i) * H; \
        const bf16_t *up_ = static_cast<const bf16_t *>(table_ptr(a.layers, (group + NG * (mg_)) * 4 + 2)) + ((int64_t)e_ * I + g_i) * H; \
        _Pragma("unroll") for (int c = 0; c < XCH; ++c) {                                              \
            gv[c] = load_global_stream<u32x4_t>(gp_ + loff + c * 512);                                       \
            uv[c] = load_global_stream<u32x4_t>(up_ + loff + c * 512);                                       \
        }                                                                                             \
        if (++g_i == I) { g_i = 0; ++g_j; }                                                           \
    }

        // Loads of iteration `itn`, requested from inside the previous iteration's stream (under load a
        // round trip to memory takes several microseconds, and an iteration that fetched and waited
        // at its start would leave the memory pipe empty that long).  The polls go out before the
        // previous iteration's down projection: what they ask for was published at least half an
        // iteration earlier.  The router segments of the layer the iteration starts and the gate / up
        // rows of the first two activations of the layer whose experts it evaluates go out last.  The selection the gate / up rows depend on was made at the start of
        // the previous iteration by one wavefront of this workgroup; its flag says whether it is
        // there.  Nobody waits for it: a wavefront that gets here first (an iteration with nothing
        // else to do) requests its rows behind the next barrier instead.
#define DP_ISSUE_POLLS(itn)                                                                           \
    {                                                                                                 \
        const int mT_ = (itn) - 1, mD_ = (itn) - 4;                                                   \
        int tid_ = threadIdx.x;                                                                       \
        asm volatile("" : "+v"(tid_));                                                                \
        if (mT_ >= 0 && mT_ < n_mine) {                                                               \
            const unsigned long long *src_ = logit_ring + (size_t)(mT_ & (DEC_RING - 1)) * n_items1;  \
            _Pragma("unroll") for (int k = 0; k < DP_POLL_L; ++k) {                                    \
                const int q_ = tid_ + k * DP_THREADS;                                                 \
                if (q_ < n_items1) pl[k] = poll_word(src_ + q_);                                      \
            }                                                                                         \
        }                                                                                             \
        if (mD_ >= 0) {                                                                               \
            const unsigned long long *src_ = h_ring + (size_t)(mD_ & (DEC_RING - 1)) * a.h_slot;      \
            _Pragma("unroll") for (int k = 0; k < DP_POLL_H; ++k) {                                    \
                const int q_ = tid_ + k * DP_THREADS;                                                 \
                if (q_ < n_words) ph[k] = poll_word(src_ + q_);                                       \
            }                                                                                         \
        }                                                                                             \
        __builtin_amdgcn_sched_barrier(0);                                                            \
    }
#define DP_ISSUE_LOADS(itn)                                                                           \
    {                                                                                                 \
        const int mR_ = (itn), mG_ = (itn) - 2;                                                       \
        int tid_ = threadIdx.x;                                                                       \
        asm volatile("" : "+v"(tid_));                                                                \
        if (mR_ < n_mine) {                                                                           \
            const float *w_router_ = static_cast<const float *>(table_ptr(a.layers, (group + NG * mR_) * 4)); \
            _Pragma("unroll") for (int r = 0; r < DP_MAX_R; ++r) {                                     \
                const int item_ = gw + r * W;                                                         \
                if (item_ < n_items1) {                                                               \
                    const int e_ = item_ / segs;                                                      \
                    const uint32_t off_ = (uint32_t)(e_ * H + (item_ - e_ * segs) * DEC_SEG) * 4u;    \
                    wr[r] = load_global<floatx4_t>(reinterpret_cast<const char *>(w_router_) + off_ + (uint32_t)(tid_ & 63) * 16u); \
                }                                                                                     \
            }                                                                                         \
        }                                                                                             \
        g_j = item0 / I;                                                                              \
        g_i = item0 - g_j * I;                                                                        \
        g_ahead = false;                                                                              \
        if (mG_ >= 0 && mG_ < n_mine && nit > 0) {                                                    \
            const uint32_t want_ = tag0 + (uint32_t)(group + NG * mG_);                               \
            const uint32_t have_ = __hip_atomic_load(&sel_tag[mG_ & (DP_SEL - 1)], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP); \
            if (__builtin_amdgcn_readfirstlane(have_) == want_) {                                     \
                DP_LOAD_ITEM(gA, uA, mG_)                                                             \
                if (nit > 1) DP_LOAD_ITEM(gB, uB, mG_)                                                \
                g_ahead = true;                                                                       \
            }                                                                                         \
        }                                                                                             \
        __builtin_amdgcn_sched_barrier(0);                                                            \
    }

        int g_j = 0, g_i = 0;     // (expert slot, intermediate index) of the next activation to load
        bool g_ahead = false;     // the first gate / up rows of the coming iteration are already requested
        if (n_mine > 0) DP_ISSUE_LOADS(0)

#pragma unroll 1
        for (int it = 0; it < (n_mine > 0 ? n_mine + 4 : 0); ++it) {
            const int mR = it, mT = it - 1, mG = it - 2, mD = it - 4;      // layer numbers inside the group
            const bool doR = mR < n_mine, doT = mT >= 0 && mT < n_mine, doG = mG >= 0 && mG < n_mine, doD = mD >= 0;
            const int lR = group + NG * mR, lT = group + NG * mT, lG = group + NG * mG, lD = group + NG * mD;

            // ---- consume the polls: partial logits of layer lT, activations of layer lD.  A word whose
            // tag is not there yet (its producer is more than a pipeline stage behind) is asked for again
            // by the wavefront that needs it, on its own, until it arrives or the wait limit passes; the
            // one workgroup barrier behind this block is the only synchronisation of the iteration -------
            {
                int tid_c = threadIdx.x;
                asm volatile("" : "+v"(tid_c));
                // the row counter of the next iteration (last used three iterations ago)
                if (tid_c == 0) row_ctr[(it + 1) & 3] = 0;
                const uint32_t tg = tag0 + (uint32_t)lT;
                const uint32_t td = tag16(tag0 + (uint32_t)lD);
                const unsigned long long *srcl = logit_ring + (size_t)(mT & (DEC_RING - 1)) * n_items1;
                const unsigned long long *srch = h_ring + (size_t)(mD & (DEC_RING - 1)) * a.h_slot;
                float *dstl = lpart[it & 1];
                bf16_t *dsth = hl[mD & 1];
                uint32_t missing = 0;                  // bit k: logit word k, bit 8 + k: activation word k
                unsigned long long t0 = 0;
                bool timing = false;
                for (;;) {
                    if (doT) {
#pragma unroll
                        for (int k = 0; k < DP_POLL_L; ++k) {
                            const int q = tid_c + k * DP_THREADS;
                            if (q < n_items1 && (!timing || (missing >> k & 1))) {
                                if ((uint32_t)(pl[k] >> 32) == tg) { dstl[q] = __uint_as_float((uint32_t)pl[k]); missing &= ~(1u << k); }
                                else missing |= 1u << k;
                            }
                        }
                    }
                    if (doD) {
#pragma unroll
                        for (int k = 0; k < DP_POLL_H; ++k) {
                            const int u = tid_c + k * DP_THREADS;         // word u: wavefront u / wpw, its word u % wpw
                            if (u < n_words && (!timing || (missing >> (8 + k) & 1))) {
                                const int wv = u / wpw, kk = u - wv * wpw;
                                const int i0 = wv * ipw + 3 * kk;          // first activation in the word
                                int nv = ipw - 3 * kk;                     // how many it holds
                                if (nv > 3) nv = 3;
                                if (nv > KI - i0) nv = KI - i0;
                                if (nv <= 0) { missing &= ~(1u << (8 + k)); }
                                else if ((uint32_t)(ph[k] >> 48) == td) {
                                    dsth[i0] = (bf16_t)ph[k];
                                    if (nv > 1) dsth[i0 + 1] = (bf16_t)(ph[k] >> 16);
                                    if (nv > 2) dsth[i0 + 2] = (bf16_t)(ph[k] >> 32);
                                    missing &= ~(1u << (8 + k));
                                } else missing |= 1u << (8 + k);
                            }
                        }
                    }
                    if (!__any(missing != 0)) break;
                    // ask again for what is missing (agent-scope loads), with the bounded wait
                    if (!timing) { t0 = wall_clock64(); timing = true; }
                    const uint32_t ab = __hip_atomic_load(a.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (ab || wall_clock64() - t0 > a.spin_limit) {
                        if (!ab) __hip_atomic_store(a.abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        if (lane == 0) behind_lds = 1;     // the workgroup leaves together behind the barrier
                        break;
                    }
#pragma unroll
                    for (int k = 0; k < DP_POLL_L; ++k)
                        if (missing >> k & 1) pl[k] = poll_word(srcl + tid_c + k * DP_THREADS);
#pragma unroll
                    for (int k = 0; k < DP_POLL_H; ++k)
                        if (missing >> (8 + k) & 1) ph[k] = poll_word(srch + tid_c + k * DP_THREADS);
                }
            }
            DP_LDS_BARRIER();
            if (behind_lds) return;        // the grid is aborting (set by a wavefront whose wait ran out)

            if (doG && nit > 0 && !g_ahead) {          // the selection was not there yet when this iteration was set up
                DP_LOAD_ITEM(gA, uA, mG)
                if (nit > 1) DP_LOAD_ITEM(gB, uB, mG)
            }

            // ---- T(lT): top-k and softmax of layer lT by the wavefront whose turn it is: K rounds of
            // wavefront maximum, ties to the lower id.  The result is first needed when the next
            // iteration's first gate / up rows are requested, at the end of this one ----------------------
            if (doT && wave == (it & (DP_WAVES - 1))) {
                const float NEG_INF = -__builtin_inff();
                const float *lp = lpart[it & 1];
                // An expert's segment products are added in segment order in runs of at most eight, then the
                // runs in order (one run up to hidden = 2048, two at 4096): the association the chained
                // kernel's per-workgroup sums have, so that both orders produce the same logits bit for bit.
                float v0 = NEG_INF, v1 = NEG_INF;
                if (lane < N) {
                    for (int r0 = 0; r0 < segs; r0 += 8) {
                        float run = 0.f;
                        for (int q = r0; q < segs && q < r0 + 8; ++q) run += lp[lane * segs + q];
                        v0 = r0 ? v0 + run : run;
                    }
                }
                if (lane + 64 < N) {
                    for (int r0 = 0; r0 < segs; r0 += 8) {
                        float run = 0.f;
                        for (int q = r0; q < segs && q < r0 + 8; ++q) run += lp[(lane + 64) * segs + q];
                        v1 = r0 ? v1 + run : run;
                    }
                }
                float m0 = v0, m1 = v1, my_z = NEG_INF, zmax = 0.f;
                int my_e = 0;
                for (int j = 0; j < K; ++j) {
                    const float m = wave_max(fmaxf(m0, m1));
                    const unsigned long long b0 = __ballot(m0 == m), b1 = __ballot(m1 == m);
                    const int e = b0 ? __ffsll((long long)b0) - 1 : 63 + __ffsll((long long)b1);
                    if (j == 0) zmax = m;
                    if (lane == j) { my_z = m; my_e = e; }
                    if (e == lane) m0 = NEG_INF;
                    if (e == lane + 64) m1 = NEG_INF;
                }
                const float den = wave_sum(((lane < N) ? expf(v0 - zmax) : 0.f) + ((lane + 64 < N) ? expf(v1 - zmax) : 0.f));
                const float my_p = (lane < K) ? expf(my_z - zmax) : 0.f;
                float wgt = my_p / den;
                if (a.renorm) wgt = my_p / wave_sum(my_p);
                if (lane < K) {
                    sel_e[mT & (DP_SEL - 1)][lane] = my_e;
                    sel_w[mT & (DP_SEL - 1)][lane] = wgt;
                    if (gr == 0) {
                        const int64_t o = ((int64_t)lT * a.steps_total + g) * K + lane;
                        a.out_idx[o] = my_e;
                        a.out_w[o] = wgt;
                    }
                }
                // LDS operations of one wavefront complete in order: the flag follows the selection
                if (lane == 0)
                    __hip_atomic_store(&sel_tag[mT & (DP_SEL - 1)], tag0 + (uint32_t)lT, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
            }

            // ---- R(lR): this wavefront's router segments (requested an iteration ago) -> tagged partial
            // logits ---------------------------------------------------------------------------------------
            if (doR) {
                unsigned long long *dstp = logit_ring + (size_t)(mR & (DEC_RING - 1)) * n_items1;
#pragma unroll
                for (int r = 0; r < DP_MAX_R; ++r) {
                    const int item = gw + r * W;
                    if (item < n_items1) {
                        const int e = item / segs;
                        const int k0 = (item - e * segs) * DEC_SEG + lane * 4;
                        const uint2 xb = *reinterpret_cast<const uint2 *>(&xs[k0]);
                        float p = wr[r].x * __uint_as_float(xb.x << 16);
                        p = fmaf(wr[r].y, __uint_as_float(xb.x & 0xFFFF0000u), p);
                        p = fmaf(wr[r].z, __uint_as_float(xb.y << 16), p);
                        p = fmaf(wr[r].w, __uint_as_float(xb.y & 0xFFFF0000u), p);
                        p = wave_sum(p);
                        if (lane == 0) put_tagged(dstp + item, p, tag0 + (uint32_t)lR);
                    }
                }
            }

            // ---- statistics of layer lG (one wavefront of the group), riding on the loads in flight ------
            if (doG && stats_wave) online_trace_stats(a, ts, lG, g, sel_e[mG & (DP_SEL - 1)], lane);

            // Takes the next output row of this workgroup's share of layer lD off the shared counter:
            // rows go to whichever wavefront is free, so the wavefronts of a workgroup reach the next
            // barrier together however unevenly memory served them during the gate / up phase.
            const int nD = doD ? wg_rows : 0;
            uint32_t *ctr = &row_ctr[it & 3];
#define DP_GRAB_ROW(r)                                                                                \
    {                                                                                                 \
        uint32_t got_ = 0;                                                                            \
        if (lane == 0) got_ = __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); \
        r = __builtin_amdgcn_readfirstlane((int)got_);                                                \
    }
            int rA = nD, rB = nD;
            bool d_issued = false;
#define DP_ISSUE_D01()                                                                                \
    if (!d_issued) {                                                                                  \
        if (it + 1 < n_mine + 4) { DP_ISSUE_POLLS(it + 1) }                                           \
        if (nD > 0) {                                                                                 \
            DP_GRAB_ROW(rA)                                                                           \
            DP_GRAB_ROW(rB)                                                                           \
            __builtin_amdgcn_sched_barrier(0);    /* the loop counts on A's loads preceding B's */     \
            DP_LOAD_DROW(dvA, mD, wg_row0 + rA, rA < nD)                                              \
            __builtin_amdgcn_sched_barrier(0);                                                        \
            DP_LOAD_DROW(dvB, mD, wg_row0 + rB, rB < nD)                                              \
            __builtin_amdgcn_sched_barrier(0);                                                        \
        } else {                          /* defined on every path: no register is kept for them */   \
            _Pragma("unroll") for (int c = 0; c < DCH; ++c) { dvA[c] = u32x4_t{0, 0, 0, 0}; dvB[c] = u32x4_t{0, 0, 0, 0}; } \
        }                                                                                             \
        d_issued = true;                                                                              \
    }

            // ---- G(lG): roll over this wavefront's activations of layer lG; the gate / up rows of the
            // first two are in flight since the previous iteration, register sets A and B alternate.
            // Every third activation closes an exchange word.  The first output rows of D are requested
            // before the last activation is reduced ---------------------------------------------------------
            {
                const int nG = doG ? nit : 0;
                const unsigned long long h_tag = (unsigned long long)tag16(tag0 + (uint32_t)lG) << 48;
                unsigned long long h_word = h_tag;
                const bf16_t *xcur = xs;
#define DP_REDUCE_ITEM(gv, uv, u)                                                                     \
    {                                                                                                 \
        float gs_ = 0.f, us_ = 0.f;                                                                   \
        _Pragma("unroll") for (int c = 0; c < XCH; ++c) {                                              \
            const u32x4_t xq_ = *reinterpret_cast<const u32x4_t *>(&xcur[(c * 64 + lane) * 8]);       \
            gs_ = dot8_bf16(gv[c], xq_, gs_);                                                         \
            us_ = dot8_bf16(uv[c], xq_, us_);                                                         \
        }                                                                                             \
        gs_ = wave_sum(gs_);                                                                          \
        us_ = wave_sum(us_);                                                                          \
        const int sub_ = (u) % 3;                                                                     \
        h_word |= (unsigned long long)f32_to_bf16(gs_ / (1.0f + expf(-gs_)) * us_) << (16 * sub_);    \
        if (sub_ == 2 || (u) == nG - 1) {                                                             \
            if (lane == 0)                                                                            \
                __hip_atomic_store(&h_ring[(size_t)(mG & (DEC_RING - 1)) * a.h_slot + gw * wpw + (u) / 3], h_word, \
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);                       \
            h_word = h_tag;                                                                           \
        }                                                                                             \
    }
                int u = 0;
#pragma unroll 1
                for (; u + 3 < nG; u += 2) {                   // steady state: both sets are refilled, no branch
                    DP_REDUCE_ITEM(gA, uA, u)
                    DP_LOAD_ITEM(gA, uA, mG)
                    DP_REDUCE_ITEM(gB, uB, u + 1)
                    DP_LOAD_ITEM(gB, uB, mG)
                }
#pragma unroll 1
                for (; u < nG; u += 2) {                       // the last activations
                    if (u + 1 >= nG) { DP_ISSUE_D01() }        // u is the last activation
                    DP_REDUCE_ITEM(gA, uA, u)
                    if (u + 2 < nG) DP_LOAD_ITEM(gA, uA, mG)
                    if (u + 1 < nG) {
                        if (u + 2 >= nG) { DP_ISSUE_D01() }    // u + 1 is the last activation
                        DP_REDUCE_ITEM(gB, uB, u + 1)
                        if (u + 3 < nG) DP_LOAD_ITEM(gB, uB, mG)
                    }
                }
                DP_ISSUE_D01()
            }

            // ---- D(lD): output rows of layer lD, taken one at a time off the workgroup's counter; the
            // two register sets alternate, a set is refilled as soon as its row is reduced.  Row numbers
            // come off the counter in order, so once a set draws a number past the end every later draw
            // does too ------------------------------------------------------------------------------------
            {
                const bf16_t *hcur = hl[mD & 1];
                const float *sw_d = sel_w[mD & (DP_SEL - 1)];
#define DP_REDUCE_DROW(dv, r_)                                                                        \
    {                                                                                                 \
        int lane_d = threadIdx.x & 63;                                                                \
        asm volatile("" : "+v"(lane_d));                                                              \
        float acc = 0.f;                                                                              \
        _Pragma("unroll") for (int c = 0; c < DCH; ++c) {                                              \
            const int q = c * 64 + lane_d;                                                            \
            const int qc = q < dchunks ? q : dchunks - 1;                                             \
            const u32x4_t hq = *reinterpret_cast<const u32x4_t *>(&hcur[qc * 8]);                     \
            const float w_ = q < dchunks ? sw_d[DP_SLOT_OF(qc)] : 0.f;                                \
            acc = fmaf(w_, dot8_bf16(dv[c], hq, 0.f), acc);                                           \
        }                                                                                             \
        acc = wave_sum(acc);                                                                          \
        if (lane == 0 && (r_) < nD) a.y[(g * L + lD) * H + wg_row0 + (r_)] = f32_to_bf16(acc);        \
    }
#pragma unroll 1
                while (rA < nD) {                  // one exit: a set that drew no row costs one idle pass
                    DP_REDUCE_DROW(dvA, rA)
                    DP_GRAB_ROW(rA)
                    DP_LOAD_DROW(dvA, mD, wg_row0 + rA, rA < nD)
                    DP_REDUCE_DROW(dvB, rB)
                    DP_GRAB_ROW(rB)
                    DP_LOAD_DROW(dvB, mD, wg_row0 + rB, rB < nD)
                }
            }

            // ---- the next iteration's first weight rows go out before this wavefront goes to the
            // barrier: the memory pipe stays busy while the workgroup gathers ------------------------------
            if (it + 1 < n_mine + 4) { DP_ISSUE_LOADS(it + 1) }
        }

        // ---- the step is complete everywhere before the next one starts ---------------------------------
        if (!grid_barrier(a, ++bar_phase, &bar_ok)) return;
    }

    if (gr == GS - 1) {                                  // trace state back to device memory
        __syncthreads();
        for (int q = tid; q < n_mine * 128; q += DP_THREADS) {
            const int l = group + NG * (q >> 7), e = q & 127;
            if (e < N) a.lru_state[l * N + e] = ts.last[l][e];
        }
        for (int q = tid; q < n_mine; q += DP_THREADS) {
            const int l = group + NG * q;
            a.sum_overlap[l] = ts.sum_ov[l];
            for (int c = 0; c < a.n_caps; ++c) {
                a.total_miss[c * L + l] = ts.tot[c][l];
                a.bytes_fetched[c * L + l] = ts.tot[c][l] * a.expert_bytes;
            }
        }
    }
}

__global__ void decode_pipe_clear(uint32_t *bar, int n, uint32_t *abort_flag, unsigned long long *tagged, int n_tagged)
{
    for (int q = threadIdx.x; q < n; q += blockDim.x) bar[q] = 0u;
    for (int q = threadIdx.x; q < n_tagged; q += blockDim.x) tagged[q] = 0ull;   // tag 0 = no layer-step
    if (threadIdx.x == 0) *abort_flag = 0u;
}

}  // namespace

remoe_status launch_decode_pipelined(const DecodeLaunch &d, hipStream_t stream)
{
    if (d.H != 512 && d.H != 1024 && d.H != 2048 && d.H != 4096)
        return fail(REMOE_E_UNSUPPORTED, "decode supports hidden in {512, 1024, 2048, 4096} (got %d)", d.H);
    if (d.I % 8 != 0 || d.K * d.I > DP_MAX_KI)
        return fail(REMOE_E_UNSUPPORTED, "decode needs inter %% 8 == 0 and top_k * inter <= %d", DP_MAX_KI);
    if (d.n_layers > DEC_MAX_LAYERS)
        return fail(REMOE_E_UNSUPPORTED, "decode keeps the trace state of at most %d layers (got %d)", DEC_MAX_LAYERS, d.n_layers);
    if (d.n_caps < 0 || d.n_caps > DEC_MAX_CAPS)
        return fail(REMOE_E_INVALID_ARG, "n_caps %d outside 0..%d", d.n_caps, DEC_MAX_CAPS);
    if ((int64_t)d.N * d.H * d.I * 2 >= ((int64_t)1 << 32))
        return fail(REMOE_E_UNSUPPORTED, "decode: one layer's down-projection tensor spans 4 GiB or more");
    if ((int64_t)d.steps_total * d.n_layers + d.n_layers >= ((int64_t)1 << 32))
        return fail(REMOE_E_UNSUPPORTED, "decode: steps_total * n_layers does not fit the 32-bit exchange tags");
    int dev = 0, n_cu = 0;
    REMOE_HIP_TRY(hipGetDevice(&dev));
    REMOE_HIP_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
    if (n_cu < 1) return fail(REMOE_E_HIP, "device reports no compute units");
    const int G = n_cu;
    const int NG = (G % DP_GROUPS == 0) ? DP_GROUPS : 1;
    const int W = (G / NG) * DP_WAVES;                   // wavefronts per group
    const DecodeWsLayout wl = decode_ws_layout(d.H, d.N, d.I, d.K);
    if (G > DEC_MAX_GRID) return fail(REMOE_E_UNSUPPORTED, "decode: %d compute units exceed the barrier's %d flags", G, DEC_MAX_GRID);
    const int ipw = (d.K * d.I + W - 1) / W;
    const int n_words = W * ((ipw + 2) / 3);
    if (n_words > DP_POLL_H * DP_THREADS || n_words > wl.n_h)
        return fail(REMOE_E_UNSUPPORTED, "decode: %d exchange words per layer exceed the %d a workgroup polls", n_words,
                    DP_POLL_H * DP_THREADS);
    const int n_seg = d.N * (d.H / DEC_SEG);
    if (n_seg > DP_POLL_L * DP_THREADS || n_seg > DP_MAX_R * W)
        return fail(REMOE_E_UNSUPPORTED, "decode: n_experts * hidden / 256 = %d router segments are more than %d wavefronts x %d",
                    n_seg, W, DP_MAX_R);

    PipeArgs a;
    a.layers = d.layers;
    a.x = static_cast<const bf16_t *>(d.x);
    a.steps_total = d.steps_total;
    a.step0 = d.step0;
    a.n_steps = d.n_steps;
    a.n_layers = d.n_layers;
    a.H = d.H; a.N = d.N; a.I = d.I; a.K = d.K; a.renorm = d.renorm;
    a.y = static_cast<bf16_t *>(d.y);
    a.out_idx = d.out_idx;
    a.out_w = d.out_w;
    a.n_caps = d.n_caps;
    for (int c = 0; c < DEC_MAX_CAPS; ++c) a.caps[c] = (c < d.n_caps) ? d.caps[c] : 0;
    a.expert_bytes = d.expert_bytes;
    a.lru_state = d.lru_state;
    a.out_overlap = d.out_overlap;
    a.out_miss = d.out_miss;
    a.sum_overlap = reinterpret_cast<unsigned long long *>(d.sum_overlap);
    a.total_miss = reinterpret_cast<unsigned long long *>(d.total_miss);
    a.bytes_fetched = reinterpret_cast<unsigned long long *>(d.bytes_fetched);
    char *ws = static_cast<char *>(d.workspace);
    a.abort_flag = reinterpret_cast<uint32_t *>(ws + 128);
    a.bar = reinterpret_cast<uint32_t *>(ws + 256);
    a.logit_ring = reinterpret_cast<unsigned long long *>(ws + wl.logit_off);
    a.h_ring = reinterpret_cast<unsigned long long *>(ws + wl.h_off);
    a.h_slot = wl.n_h;
    a.spin_limit = d.spin_limit_ticks;

    // both ring regions are contiguous from logit_off to the end of the workspace
    hipLaunchKernelGGL(decode_pipe_clear, dim3(1), dim3(1024), 0, stream, a.bar, G, a.abort_flag, a.logit_ring,
                       (int)((wl.total - wl.logit_off) / sizeof(unsigned long long)));
    void *params[] = {&a};
    const void *fn = nullptr;
    const bool few = d.K * d.I <= 4 * 512;               // down-row chunks per lane: 4 or DP_MAX_DCH
    switch (d.H / 512) {
    case 1: fn = few ? reinterpret_cast<const void *>(decode_pipe_kernel<1, 4>) : reinterpret_cast<const void *>(decode_pipe_kernel<1, DP_MAX_DCH>); break;
    case 2: fn = few ? reinterpret_cast<const void *>(decode_pipe_kernel<2, 4>) : reinterpret_cast<const void *>(decode_pipe_kernel<2, DP_MAX_DCH>); break;
    case 4: fn = few ? reinterpret_cast<const void *>(decode_pipe_kernel<4, 4>) : reinterpret_cast<const void *>(decode_pipe_kernel<4, DP_MAX_DCH>); break;
    case 8: fn = few ? reinterpret_cast<const void *>(decode_pipe_kernel<8, 4>) : reinterpret_cast<const void *>(decode_pipe_kernel<8, DP_MAX_DCH>); break;
    default: return fail(REMOE_E_UNSUPPORTED, "decode supports hidden in {512, 1024, 2048, 4096} (got %d)", d.H);
    }
    // Every workgroup must be resident (the exchanges and the step barrier wait for all of them): one
    // workgroup per compute unit, checked against the occupancy; unused dynamic LDS lifts a workgroup
    // above half a compute unit's 160 KB so that no two share a compute unit while another idles.
    hipFuncAttributes attr;
    REMOE_HIP_TRY(hipFuncGetAttributes(&attr, fn));
    const size_t half_lds = 80 * 1024 + 256;
    const size_t pad = attr.sharedSizeBytes < half_lds ? half_lds - attr.sharedSizeBytes : 0;
    int per_cu = 0;
    REMOE_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, DP_THREADS, pad));
    if (per_cu < 1) return fail(REMOE_E_UNSUPPORTED, "decode: a workgroup does not fit one compute unit");
    REMOE_HIP_TRY(hipLaunchKernel(fn, dim3(G), dim3(DP_THREADS), params, pad, stream));
    return REMOE_OK;
}

}  // namespace remoe
