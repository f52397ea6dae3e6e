// M = 1 decode with the layers chained: the whole MoE layer for one token per step, weights streamed
// once from HBM, a layer starting only when the previous one has finished on every compute unit.
//
// At one token per step the layer (Sec. 3.1 routing, Sec. 4.1 step 5 expert execution) is a chain
// of matrix-vector products with about one flop per byte, so the matrix cores are useless and the
// only roofline is HBM bandwidth: per layer-step the fp32 router matrix (N_r x H) and the three
// matrices of the K selected experts are read exactly once (the B = 1 regime of Sec. 3).  What
// stands between a kernel and that roofline is the chain of dependencies inside a layer and from
// one layer to the next, which a decoder cannot reorder:
//
//     output of layer l-1 complete  ->  router logits of layer l  ->  top-k  ->  gate/up rows of the
//     selected experts  ->  SwiGLU activations h complete  ->  down rows  ->  output of layer l
//
// Three of these arrows are exchanges between ALL compute units (every logit needs the whole input
// row, the top-k needs every logit, every output row needs all of h).  One persistent kernel runs
// all layers of all steps of a call, one workgroup per compute unit, and is organised so that HBM
// keeps streaming across those exchanges wherever the data dependencies allow it:
//
//   * A workgroup has 8 streaming wavefronts and one exchange wavefront.  Vector-memory loads
//     return to a wavefront in the order it issued them, so a wavefront with 30 KB of weights on
//     their way cannot see an exchange word before all of them have arrived.  The exchange
//     wavefront never loads weights: it polls the words the other workgroups publish (agent-scope
//     loads, which bypass the per-XCD L2), hands the result over through LDS, and meets its
//     workgroup's streaming wavefronts at LDS-only workgroup barriers (a full barrier would also
//     wait for every weight load in flight).
//   * Exchanged values carry the number of the layer-step that produced them as a tag (a partial
//     logit: fp32 + 32-bit tag; up to three bf16 values of one wavefront + a 16-bit tag in one
//     8-byte word), so a reader needs no separate flag: it polls until the tags match.  Every
//     value is published once per XCD (eight copies, one store instruction), and a workgroup polls
//     its own XCD's copy: 32 readers per copy instead of 256 on the same few memory channels.
//   * As soon as the selection of a layer is known, a streaming wavefront requests its router
//     segment of the NEXT layer (the only data of the next layer that does not depend on this
//     layer's output) and the gate and up rows of all three of its activations (three register
//     sets).  Its row of the down projection, from all K experts, is requested as soon as its
//     activations are published: every wavefront's gate / up rows are then ahead of every down row
//     in the memory system's queues, and the down rows are on their way while h is being
//     exchanged.  The loops are straight-line code with a fixed number of loads, so the compiler's
//     wait counts let one set be reduced while the later requests stay in flight.
//   * A layer ends with every wavefront publishing its output value(s); the exchange wavefronts
//     gather them all (in a decoder they are the next layer's input row) before the router
//     products of the next layer are formed from the prefetched router segments.  The same gather
//     closes a step, so there is no separate grid barrier anywhere.
//
// The top-k / softmax of a layer is computed by the exchange wavefront of every workgroup (same
// result everywhere: K rounds of wavefront maximum, ties to the lower id).  The routing-trace
// statistics the paper optimises are updated online by the exchange wavefront of the last
// workgroup right after its top-k: the adjacent-step overlap |E_t n E_{t-1}| (Eq. 1) and the LRU
// misses |E_t \ C_t| (App. E.2) for up to four cache capacities from one per-expert "last used"
// table per layer.
//
// SwiGLU activations cross workgroups as bf16 (what the batched path stores between its two GEMMs as
// well), gate/up and down products are packed bf16 dot instructions with fp32 accumulation, the same
// arithmetic in the same order as the layer-overlapped kernel (decode_pipe.hip), so both orders
// give the same bits.
//
// Every wait is bounded: an exchange wavefront that waits longer than the limit raises the abort
// word, every other one sees it in its next poll, and each workgroup leaves together at its next
// barrier.
#include "common.h"
#include "decode_common.h"
#include "topk.h"

namespace remoe {

namespace {

constexpr int CH_STREAM = 8;                          // streaming wavefronts per workgroup
constexpr int CH_WAVES = CH_STREAM + 1;               // + the exchange wavefront
constexpr int CH_THREADS = CH_WAVES * 64;
constexpr int CH_MAX_KI = 6144;                       // K * I activations of one layer
constexpr int CH_ITEMS = 3;                           // activations per streaming wavefront (at most)
constexpr int CH_MAX_R = 1;                           // router segments per streaming wavefront (at most)
constexpr int CH_POLL = 32;                           // exchange words per lane and polling pass

struct ChainArgs {
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
    uint32_t *lru_state;         // [L, N] last use (global step + 1), 0 = never
    uint8_t *out_overlap;        // [L, T_total]
    uint8_t *out_miss;           // [n_caps, L, T_total]
    unsigned long long *sum_overlap;   // [L]
    unsigned long long *total_miss;    // [n_caps, L]
    unsigned long long *bytes_fetched; // [n_caps, L]
    unsigned long long *logit_x;  // [copies] x logit_stride words: (tag << 32) | float bits, one per router segment
    unsigned long long *h_x;      // [copies] x word_stride words: 3 x bf16 | tag16 << 48, activations
    unsigned long long *y_x;      // [copies] x word_stride words: 3 x bf16 | tag16 << 48, output values
    int logit_stride, word_stride;
    uint32_t *abort_flag;        // zero at launch
    unsigned long long spin_limit;   // wall-clock ticks (100 MHz) a single wait may last
};

// Workgroup barrier that orders LDS traffic only (a full __syncthreads would also wait for every
// weight load in flight, which is exactly what must keep flying).
#define CH_LDS_BARRIER() asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory")

// 16-bit tag of a layer-step (never 0, the value of a cleared word).  A word is rewritten every
// layer-step, so one that is 65535 layer-steps old cannot survive to be mistaken for a new one.
__device__ __forceinline__ uint32_t ch_tag16(uint32_t tag) { return tag % 65535u + 1u; }

__device__ __forceinline__ unsigned long long ch_poll(const unsigned long long *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// One 8-byte word into every XCD's copy of an exchange array: lane c of the wavefront stores copy c.
__device__ __forceinline__ void ch_publish(unsigned long long *base, int stride, int copies, int index,
                                           unsigned long long word, int lane)
{
    if (lane < copies)
        __hip_atomic_store(base + (size_t)lane * stride + index, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Exchange wavefront: polls words [0, n) of `src` until every one carries `tag16` in its top 16 bits,
// then hands each to `sink(index, word)`.  All polls of a pass of up to 64 x CH_POLL words are in
// flight together; the pass is repeated until every word is there, the abort word is raised or the
// wait limit passes.  Returns false when the grid is aborting.
template <class Sink>
__device__ __forceinline__ bool ch_gather16(const ChainArgs &a, const unsigned long long *src, int n, uint32_t tag16,
                                            Sink sink)
{
    // (the lane number is taken from a value the optimiser cannot see through, so that the poll addresses
    // are formed here from one base and constant offsets instead of being kept in registers for the
    // whole kernel)
    int lane = threadIdx.x & 63;
    asm volatile("" : "+v"(lane));
    for (int base = 0; base < n; base += 64 * CH_POLL) {
        // Words past n are read as well (the launcher keeps 64 x CH_POLL words readable behind every array)
        // and simply not looked at: every lane then polls base + lane + 64 k for constant k.  A pass that
        // finds a word missing is repeated as a whole after a short pause: straight-line code, and with the
        // wait for the own workgroup in front of it a repeat is the exception.
        const unsigned long long *p = src + base + lane;
        unsigned long long w[CH_POLL];
        unsigned long long t0 = 0;
        bool timing = false;
        for (;;) {
#pragma unroll
            for (int k = 0; k < CH_POLL; ++k) w[k] = ch_poll(p + k * 64);
            bool missing = false;
#pragma unroll
            for (int k = 0; k < CH_POLL; ++k)
                missing |= base + k * 64 + lane < n && (uint32_t)(w[k] >> 48) != tag16;
            if (!__any(missing)) break;
            if (!timing) { t0 = wall_clock64(); timing = true; }
            const uint32_t ab = __hip_atomic_load(a.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (ab || wall_clock64() - t0 > a.spin_limit) {
                if (!ab) __hip_atomic_store(a.abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                return false;
            }
            __builtin_amdgcn_s_sleep(4);
        }
#pragma unroll
        for (int k = 0; k < CH_POLL; ++k) {
            const int q = base + k * 64 + lane;
            if (q < n) sink(q, w[k]);
        }
    }
    return true;
}

// XCH: 16-byte chunks per lane of one hidden row (hidden / 512).  DCH: 16-byte chunks per lane of one
// down-projection output row over the K selected experts (K * inter / 512, rounded up to a supported
// count).  RPW: output rows per streaming wavefront.  All three fix the number of loads per unit of
// work at compile time.
template <int XCH, int DCH, int RPW>
__global__ __launch_bounds__(CH_THREADS) void decode_chain_kernel(const ChainArgs a)
{
    __shared__ __attribute__((aligned(16))) bf16_t hl[CH_MAX_KI];   // activations of the layer (bf16)
    __shared__ __attribute__((aligned(16))) bf16_t xs[4096];        // the step's input row
    __shared__ int sel_e[8];
    __shared__ float sel_w[8];
    __shared__ int leave_lds;            // set by the exchange wavefront when a wait ran out: the workgroup returns
    __shared__ uint32_t arrivals;        // publications of this workgroup's streaming wavefronts so far (3 per layer-step each)
    __shared__ float lp[CH_STREAM];      // router products of this workgroup's streaming wavefronts (one segment each)
    __shared__ bf16_t ys[CH_STREAM * RPW];   // output values of this workgroup's streaming wavefronts
    __shared__ unsigned long long wtab[DEC_MAX_LAYERS * 4];   // the launch's weight-pointer table
    __shared__ TraceLds ts;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool exchange = wave == CH_STREAM;
    const int G = gridDim.x;
    const int copies = (G % DEC_GROUPS == 0) ? DEC_GROUPS : 1;   // workgroup b runs on XCD b % 8 and polls that copy
    const int my_copy = blockIdx.x % copies;
    const int W = G * CH_STREAM;                                   // streaming wavefronts in the grid
    const int gw = blockIdx.x * CH_STREAM + wave;                  // this streaming wavefront's index
    const int H = a.H, N = a.N, I = a.I, K = a.K, L = a.n_layers;
    const int segs = H / DEC_SEG;
    const int KI = K * I;
    const int n_items1 = N * segs;                  // router work items: (expert, 256-wide segment)
    const int ipw = (KI + W - 1) / W;               // activations per streaming wavefront (<= CH_ITEMS)
    const int wpw = (ipw + 2) / 3;                  // exchange words per streaming wavefront
    const int n_hwords = W * wpw;
    constexpr int YW = (CH_STREAM * RPW + 2) / 3;   // exchange words of a workgroup's output values (3 per word)
    const int n_ywords = G * YW;
    const int lgs = segs < CH_STREAM ? segs : CH_STREAM;   // router segments summed into one exchange word
    const int lwpe = segs / lgs;                    // exchange words per expert (1, or 2 when hidden = 4096)
    const int dchunks = KI / 8;
    const int chunks_per_row = I / 8;
    const bool stats_wave = blockIdx.x == G - 1 && exchange;
    const unsigned long long *const my_logits = a.logit_x + (size_t)my_copy * a.logit_stride;
    const unsigned long long *const my_h = a.h_x + (size_t)my_copy * a.word_stride;
    const unsigned long long *const my_y = a.y_x + (size_t)my_copy * a.word_stride;
    // chunk q of a wavefront's down-row work is chunk q % chunks_per_row of expert slot q / chunks_per_row;
    // the quotient by multiplication (exact for q < 2^16, chunks_per_row <= 2^16)
    const uint32_t cpr_magic = (uint32_t)((0x100000000ull + (unsigned)chunks_per_row - 1) / (unsigned)chunks_per_row);
#define CH_SLOT_OF(q) ((int)__umulhi((uint32_t)(q), cpr_magic))

    if (blockIdx.x == G - 1) {                      // trace state -> LDS
        for (int q = tid; q < L * 128; q += CH_THREADS) {
            const int l = q >> 7, e = q & 127;
            ts.last[l][e] = (e < N) ? a.lru_state[l * N + e] : 0u;
        }
        for (int q = tid; q < L; q += CH_THREADS) {
            ts.sum_ov[q] = a.sum_overlap[q];
            for (int c = 0; c < a.n_caps; ++c) ts.tot[c][q] = a.total_miss[c * L + q];
        }
    }
    if (tid == 0) { leave_lds = 0; arrivals = 0u; }
    // the weight pointers of all layers -> LDS (a read from there costs a tenth of a scalar load from memory,
    // and four of those in a row stood between the selection and the first weight request)
    for (int q = tid; q < L * 4; q += CH_THREADS) wtab[q] = reinterpret_cast<const unsigned long long *>(a.layers)[q];
    __syncthreads();
#define CH_WPTR(idx) reinterpret_cast<const void *>(((unsigned long long)__builtin_amdgcn_readfirstlane((int)(wtab[idx] >> 32)) << 32) | (unsigned)__builtin_amdgcn_readfirstlane((int)(uint32_t)wtab[idx]))
    uint32_t arrivals_due = 0;           // exchange wavefront: the count `arrivals` reaches with the next publication round

    // ---- per-wavefront constants of the streaming wavefronts ----------------------------------------
    const int item0 = gw * ipw;                     // first activation (expert slot j = item / I, index i = item % I)
    const int row0 = gw * RPW;                      // first output row

    // router segments of the layer-step that comes next, requested a layer ahead (streaming wavefronts)
    floatx4_t wr[CH_MAX_R];
#pragma unroll
    for (int r = 0; r < CH_MAX_R; ++r) wr[r] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#define CH_LOAD_ROUTER(layer_)                                                                        \
    {                                                                                                 \
        const float *w_router_ = static_cast<const float *>(CH_WPTR((layer_) * 4));                   \
        _Pragma("unroll") for (int r = 0; r < CH_MAX_R; ++r) {                                         \
            const int item_ = gw + r * W;                                                             \
            if (item_ < n_items1) {                                                                   \
                const int e_ = item_ / segs;                                                          \
                const uint32_t off_ = (uint32_t)(e_ * H + (item_ - e_ * segs) * DEC_SEG) * 4u;        \
                wr[r] = load_global<floatx4_t>(reinterpret_cast<const char *>(w_router_) + off_ + (uint32_t)lane * 16u); \
            }                                                                                         \
        }                                                                                             \
    }
    if (!exchange) CH_LOAD_ROUTER(0)

    // A streaming wavefront has published its words of a round (router products, activations or output
    // values): one LDS increment.  The exchange wavefront polls the other workgroups' words only once its
    // own workgroup's eight have published: compute units run a layer-step in near lockstep, so until
    // then most words are missing everywhere, and 256 wavefronts re-polling them would load the same
    // memory channels the weights stream through.
#define CH_ARRIVE() { if (lane == 0) __hip_atomic_fetch_add(&arrivals, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); }
#define CH_AWAIT_OWN(ok_)                                                                             \
    {                                                                                                 \
        arrivals_due += CH_STREAM;                                                                    \
        unsigned long long t0_ = 0;                                                                   \
        bool timing_ = false;                                                                         \
        while ((int32_t)(__hip_atomic_load(&arrivals, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) - arrivals_due) < 0) { \
            __builtin_amdgcn_s_sleep(2);                                                              \
            if (!timing_) { t0_ = wall_clock64(); timing_ = true; }                                   \
            else if (wall_clock64() - t0_ > a.spin_limit) {                                           \
                __hip_atomic_store(a.abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);     \
                ok_ = false;                                                                          \
                break;                                                                                \
            }                                                                                         \
        }                                                                                             \
    }

#pragma unroll 1
    for (int64_t s = 0; s < a.n_steps; ++s) {
        const int64_t g = a.step0 + s;
        const bf16_t *xg = a.x + g * H;
        // The step's input row -> LDS.  Its last readers (the gate / up products of the previous step's last
        // layer) are behind that layer's activation barrier, which every wavefront has passed.
        for (int k = tid; k < H / 8; k += CH_THREADS)
            *reinterpret_cast<u32x4_t *>(&xs[k * 8]) = *reinterpret_cast<const u32x4_t *>(xg + k * 8);

#pragma unroll 1
        for (int layer = 0; layer < L; ++layer) {
            const uint32_t n_ls = (uint32_t)(g * L + layer);      // number of this layer-step in the run
            const uint32_t tag = n_ls + 1u;                       // 32-bit tag of its partial logits
            const uint32_t t16 = ch_tag16(tag);                   // 16-bit tag of its activations and outputs
            const bool first_of_launch = s == 0 && layer == 0;

            // ---- 1. the previous layer-step is complete everywhere: the exchange wavefront gathers every
            // output value of it (a decoder's next input row) ---------------------------------------------
            if (exchange && !first_of_launch) {
                const uint32_t prev16 = ch_tag16(tag - 1u);
                bool ok = true;
                CH_AWAIT_OWN(ok)
                // this workgroup's output values of the previous layer-step (LDS) -> YW words in every copy
                if (ok && lane < YW * copies) {
                    const int k = lane / copies, cpy = lane - k * copies;
                    unsigned long long word = (unsigned long long)prev16 << 48;
#pragma unroll
                    for (int v = 0; v < 3; ++v)
                        if (3 * k + v < CH_STREAM * RPW) word |= (unsigned long long)ys[3 * k + v] << (16 * v);
                    __hip_atomic_store(a.y_x + (size_t)cpy * a.word_stride + blockIdx.x * YW + k, word, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                }
                if (ok) ok = ch_gather16(a, my_y, n_ywords, prev16, [](int, unsigned long long) {});
                if (!ok && lane == 0) leave_lds = 1;
            }
            CH_LDS_BARRIER();
            if (leave_lds) return;

            // ---- 2. router: the streaming wavefronts dot their prefetched segments with the input row -------
            if (!exchange) {
#pragma unroll
                for (int r = 0; r < CH_MAX_R; ++r) {
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
                        if (lane == 0) lp[wave] = p;
                    }
                }
                CH_ARRIVE()
            } else {
                // ---- 3. the exchange wavefront gathers the partial logits (lane l: experts l and l + 64, whose
                // segments are adjacent words), sums them in segment order, ranks them: K rounds of wavefront
                // maximum, ties to the lower id; softmax weights --------------------------------------------------
                const float NEG_INF = -__builtin_inff();
                float v0 = NEG_INF, v1 = NEG_INF;
                bool ok = true;
                CH_AWAIT_OWN(ok)
                // This workgroup's eight router products are in LDS (streaming wavefront w holds item b * 8 + w,
                // items of one expert are adjacent): sum each run of `lgs` of them in segment order and publish
                // one word per run -- an eighth of the words every workgroup would otherwise have to poll.
                if (ok && blockIdx.x * CH_STREAM < n_items1) {
                    const int runs = CH_STREAM / lgs;
                    if (lane < runs * copies) {
                        const int run = lane / copies, cpy = lane - run * copies;
                        float v = 0.f;
                        for (int q = 0; q < lgs; ++q) v += lp[run * lgs + q];
                        __hip_atomic_store(a.logit_x + (size_t)cpy * a.logit_stride + blockIdx.x * runs + run,
                                           ((unsigned long long)tag << 32) | __float_as_uint(v), __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
                if (ok) {
                    int lane_p = threadIdx.x & 63;
                    asm volatile("" : "+v"(lane_p));               // addresses formed here, not kept across the kernel
                    const unsigned long long *p0 = my_logits + lane_p * lwpe;      // expert lane: words p0[0 .. lwpe)
                    const unsigned long long *p1 = p0 + 64 * lwpe;                  // expert lane + 64
                    const bool has0 = lane_p < N, has1 = lane_p + 64 < N;
                    unsigned long long pw0[2], pw1[2];
                    unsigned long long t0 = 0;
                    bool timing = false;
                    for (;;) {                 // the whole pass is repeated when a word is missing, as in ch_gather16
                        pw0[0] = pw0[1] = pw1[0] = pw1[1] = 0ull;
                        if (has0) {
                            pw0[0] = ch_poll(p0);
                            if (lwpe > 1) pw0[1] = ch_poll(p0 + 1);
                        }
                        if (has1) {
                            pw1[0] = ch_poll(p1);
                            if (lwpe > 1) pw1[1] = ch_poll(p1 + 1);
                        }
                        bool missing = false;
#pragma unroll
                        for (int q = 0; q < 2; ++q) {
                            missing |= has0 && q < lwpe && (uint32_t)(pw0[q] >> 32) != tag;
                            missing |= has1 && q < lwpe && (uint32_t)(pw1[q] >> 32) != tag;
                        }
                        if (!__any(missing)) break;
                        if (!timing) { t0 = wall_clock64(); timing = true; }
                        const uint32_t ab = __hip_atomic_load(a.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        if (ab || wall_clock64() - t0 > a.spin_limit) {
                            if (!ab) __hip_atomic_store(a.abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            ok = false;
                            break;
                        }
                        __builtin_amdgcn_s_sleep(4);
                    }
                    if (has0) {
                        v0 = __uint_as_float((uint32_t)pw0[0]);
                        if (lwpe > 1) v0 += __uint_as_float((uint32_t)pw0[1]);
                    }
                    if (has1) {
                        v1 = __uint_as_float((uint32_t)pw1[0]);
                        if (lwpe > 1) v1 += __uint_as_float((uint32_t)pw1[1]);
                    }
                }
                if (!ok) {
                    if (lane == 0) leave_lds = 1;
                } else {
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
                        sel_e[lane] = my_e;
                        sel_w[lane] = wgt;
                        if (blockIdx.x == 0) {
                            const int64_t o = ((int64_t)layer * a.steps_total + g) * K + lane;
                            a.out_idx[o] = my_e;
                            a.out_w[o] = wgt;
                        }
                    }
                }
            }
            CH_LDS_BARRIER();                   // the selection is in LDS
            if (leave_lds) return;

            if (!exchange) {
                // ---- 4. the gate and up rows of this wavefront's three activations are requested at once ------
                const bf16_t *w_gate = static_cast<const bf16_t *>(CH_WPTR(layer * 4 + 1));
                const bf16_t *w_up = static_cast<const bf16_t *>(CH_WPTR(layer * 4 + 2));
                const char *w_down = static_cast<const char *>(CH_WPTR(layer * 4 + 3));
                // the next layer-step's router segment first (it is consumed last, and every request that follows
                // is unconditional, which keeps the compiler's wait counts exact)
                {
                    int nl = layer + 1;
                    if (nl == L) nl = 0;
                    CH_LOAD_ROUTER(nl)
                }
                __builtin_amdgcn_sched_barrier(0);
                u32x4_t gA[XCH], uA[XCH], gB[XCH], uB[XCH], gC[XCH], uC[XCH], dv[DCH];
                // gate and up rows of activation number it_ of this wavefront (past the end: the layer's last
                // activation again, its value is not published)
#define CH_LOAD_ITEM(gv, uv, it_)                                                                     \
    {                                                                                                 \
        int item_ = item0 + (it_);                                                                    \
        if (item_ >= KI) item_ = KI - 1;                                                              \
        const int j_ = item_ / I, i_ = item_ - j_ * I;                                                \
        const int e_ = __builtin_amdgcn_readfirstlane(sel_e[j_]);                                     \
        const bf16_t *gp_ = w_gate + ((int64_t)e_ * I + i_) * H;                                      \
        const bf16_t *up_ = w_up + ((int64_t)e_ * I + i_) * H;                                        \
        int loff_ = (threadIdx.x & 63) * 8;                                                           \
        asm volatile("" : "+v"(loff_));                                                               \
        _Pragma("unroll") for (int c = 0; c < XCH; ++c) {                                              \
            gv[c] = load_global_stream<u32x4_t>(gp_ + loff_ + c * 512);                               \
            uv[c] = load_global_stream<u32x4_t>(up_ + loff_ + c * 512);                               \
        }                                                                                             \
    }
                // chunks [c0, c1) of output row `row` (all K experts' pieces of it); a row past the end reads the
                // tensor's first bytes
#define CH_LOAD_DROW(row, c0, c1)                                                                     \
    {                                                                                                 \
        int lane_ = threadIdx.x & 63;                                                                 \
        asm volatile("" : "+v"(lane_));   /* offsets are recomputed here, not kept in registers */     \
        _Pragma("unroll") for (int c = (c0); c < (c1); ++c) {                                          \
            int q_ = c * 64 + lane_;                          /* past the end: the last chunk again, */ \
            if (q_ >= dchunks) q_ = dchunks - 1;              /* weighted 0 when the row is reduced  */ \
            const int j_ = CH_SLOT_OF(q_);                                                            \
            uint32_t off_ = (uint32_t)(((int64_t)sel_e[j_] * H + (row)) * I * 2) + (uint32_t)(q_ - j_ * chunks_per_row) * 16u; \
            if ((row) >= H) off_ = 0;                                                                 \
            dv[c] = load_global_stream<u32x4_t>(w_down + off_);                                       \
        }                                                                                             \
    }
                const unsigned long long h_tag = (unsigned long long)t16 << 48;
                unsigned long long h_word = h_tag;
#define CH_REDUCE_ITEM(gv, uv, u)                                                                     \
    {                                                                                                 \
        int lane_ = threadIdx.x & 63;                                                                 \
        asm volatile("" : "+v"(lane_));                                                               \
        float gs_ = 0.f, us_ = 0.f;                                                                   \
        _Pragma("unroll") for (int c = 0; c < XCH; ++c) {                                              \
            const u32x4_t xq_ = *reinterpret_cast<const u32x4_t *>(&xs[(c * 64 + lane_) * 8]);        \
            gs_ = dot8_bf16(gv[c], xq_, gs_);                                                         \
            us_ = dot8_bf16(uv[c], xq_, us_);                                                         \
        }                                                                                             \
        gs_ = wave_sum(gs_);                                                                          \
        us_ = wave_sum(us_);                                                                          \
        h_word |= (unsigned long long)f32_to_bf16(gs_ / (1.0f + expf(-gs_)) * us_) << (16 * (u));     \
    }
                static_assert(CH_ITEMS == 3, "the sequence below is written out for three activations per wavefront");
                // All gate / up rows go out before any row of the down projection, on every wavefront: the memory
                // system serves requests roughly in the order they were made, and a down row requested early by a
                // wavefront that is ahead would be served before gate / up rows of one that is behind, whose
                // activation the whole grid waits for.
                CH_LOAD_ITEM(gA, uA, 0)
                __builtin_amdgcn_sched_barrier(0);
                CH_LOAD_ITEM(gB, uB, 1)
                __builtin_amdgcn_sched_barrier(0);
                CH_LOAD_ITEM(gC, uC, 2)
                __builtin_amdgcn_sched_barrier(0);
                CH_REDUCE_ITEM(gA, uA, 0)
                __builtin_amdgcn_sched_barrier(0);
                CH_REDUCE_ITEM(gB, uB, 1)
                __builtin_amdgcn_sched_barrier(0);
                CH_REDUCE_ITEM(gC, uC, 2)
                __builtin_amdgcn_sched_barrier(0);
                // one word per wavefront (ipw <= 3): activations item0 .. item0 + ipw - 1 (the reader takes no more;
                // a wavefront without activations of its own still publishes, its tag is waited for)
                ch_publish(a.h_x, a.word_stride, copies, gw * wpw, h_word, lane);
                CH_ARRIVE()
                __builtin_amdgcn_sched_barrier(0);
                // the down-projection row streams in while the activations are exchanged
                CH_LOAD_DROW(row0, 0, DCH)
                __builtin_amdgcn_sched_barrier(0);

                // ---- 6. activations of the whole layer are in LDS (exchange wavefront): down projection ----------
                CH_LDS_BARRIER();
                if (leave_lds) return;
#pragma unroll
                for (int rw = 0; rw < RPW; ++rw) {
                    const int o = row0 + rw;
                    int lane_d = threadIdx.x & 63;
                    asm volatile("" : "+v"(lane_d));       // (recomputed per row, not kept in registers across the layer)
                    float acc = 0.f;
#pragma unroll
                    for (int c = 0; c < DCH; ++c) {
                        const int q = c * 64 + lane_d;
                        const int qc = q < dchunks ? q : dchunks - 1;
                        const u32x4_t hq = *reinterpret_cast<const u32x4_t *>(&hl[qc * 8]);
                        const float w_ = q < dchunks ? sel_w[CH_SLOT_OF(qc)] : 0.f;
                        acc = fmaf(w_, dot8_bf16(dv[c], hq, 0.f), acc);
                    }
                    if (rw + 1 < RPW) {
                        __builtin_amdgcn_sched_barrier(0);
                        CH_LOAD_DROW(o + 1, 0, DCH)
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    acc = wave_sum(acc);
                    const bf16_t yb = f32_to_bf16(acc);
                    if (lane == 0) {
                        if (o < H) a.y[(g * L + layer) * H + o] = yb;
                        ys[wave * RPW + rw] = yb;
                    }
                }
                CH_ARRIVE()
            } else {
                // ---- 5. exchange wavefront: statistics of this layer-step (one wavefront of the grid), then the
                // activations of every streaming wavefront -> LDS ------------------------------------------------
                if (stats_wave) online_trace_stats(a, ts, layer, g, sel_e, lane);
                bool ok = true;
                CH_AWAIT_OWN(ok)
                if (ok) ok = ch_gather16(a, my_h, n_hwords, t16, [&](int u, unsigned long long word) {
                    const int wv = u / wpw, kk = u - wv * wpw;
                    const int i0 = wv * ipw + 3 * kk;          // first activation in the word
                    int nv = ipw - 3 * kk;                     // how many it holds
                    if (nv > 3) nv = 3;
                    if (nv > KI - i0) nv = KI - i0;
                    if (nv > 0) hl[i0] = (bf16_t)word;
                    if (nv > 1) hl[i0 + 1] = (bf16_t)(word >> 16);
                    if (nv > 2) hl[i0 + 2] = (bf16_t)(word >> 32);
                });
                if (!ok && lane == 0) leave_lds = 1;
                CH_LDS_BARRIER();
                if (leave_lds) return;
            }
        }
    }

    // the last layer-step is complete everywhere before the kernel ends (the outputs are the caller's
    // once the stream reaches the end of the call anyway; this keeps every workgroup's exit behind the
    // last use of the exchange words)
    if (blockIdx.x == G - 1) {                  // trace state back to device memory
        __syncthreads();
        for (int q = tid; q < L * 128; q += CH_THREADS) {
            const int l = q >> 7, e = q & 127;
            if (e < N) a.lru_state[l * N + e] = ts.last[l][e];
        }
        for (int q = tid; q < L; q += CH_THREADS) {
            a.sum_overlap[q] = ts.sum_ov[q];
            for (int c = 0; c < a.n_caps; ++c) {
                a.total_miss[c * L + q] = ts.tot[c][q];
                a.bytes_fetched[c * L + q] = ts.tot[c][q] * a.expert_bytes;
            }
        }
    }
}

__global__ void decode_chain_clear(uint32_t *abort_flag, unsigned long long *tagged, int n_tagged)
{
    for (int q = threadIdx.x; q < n_tagged; q += blockDim.x) tagged[q] = 0ull;   // tag 0 = no layer-step
    if (threadIdx.x == 0) *abort_flag = 0u;
}

}  // namespace

size_t decode_workspace_bytes(int H, int N, int I, int K) { return decode_ws_layout(H, N, I, K).total; }

remoe_status launch_decode(const DecodeLaunch &d, hipStream_t stream)
{
    if (d.H != 512 && d.H != 1024 && d.H != 2048 && d.H != 4096)
        return fail(REMOE_E_UNSUPPORTED, "decode supports hidden in {512, 1024, 2048, 4096} (got %d)", d.H);
    if (d.I % 8 != 0 || d.K * d.I > CH_MAX_KI)
        return fail(REMOE_E_UNSUPPORTED, "decode needs inter %% 8 == 0 and top_k * inter <= %d", CH_MAX_KI);
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
    // one workgroup per compute unit, all resident at once (checked against the occupancy below)
    const int G = n_cu;
    if (G > DEC_MAX_GRID) return fail(REMOE_E_UNSUPPORTED, "decode: %d compute units exceed the supported %d", G, DEC_MAX_GRID);
    const int W = G * CH_STREAM;
    const int KI = d.K * d.I;
    const int ipw = (KI + W - 1) / W;
    const int rpw = (d.H + W - 1) / W;
    const int n_seg = d.N * (d.H / DEC_SEG);
    const DecodeWsLayout wl = decode_ws_layout(d.H, d.N, d.I, d.K);
    if (ipw > CH_ITEMS)
        return fail(REMOE_E_UNSUPPORTED, "decode (layers chained): top_k * inter = %d is more than %d activations for each of "
                    "the %d streaming wavefronts of this device", KI, CH_ITEMS, W);
    const int rpw_t = d.H > 2048 ? 2 : 1;            // rows per wavefront the kernel is instantiated for
    if (rpw > rpw_t)
        return fail(REMOE_E_UNSUPPORTED, "decode (layers chained): hidden %d needs %d output rows per wavefront on this "
                    "device, %d supported", d.H, rpw, rpw_t);
    if (n_seg > CH_MAX_R * W || n_seg > wl.n_logit)
        return fail(REMOE_E_UNSUPPORTED, "decode (layers chained): n_experts * hidden / 256 = %d router segments are more "
                    "than %d wavefronts x %d", n_seg, W, CH_MAX_R);
    if (W > wl.n_h)
        return fail(REMOE_E_UNSUPPORTED, "decode (layers chained): %d streaming wavefronts exceed the %d exchange words "
                    "of a ring slot", W, wl.n_h);

    ChainArgs a;
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
    // The workspace holds, per group of the layer-overlapped kernel, DEC_RING slots of partial logits and
    // DEC_RING slots of activation words.  This kernel uses, per XCD copy, the first slot of a group's
    // logit ring, and the first two slots of its word ring (activations, output values).
    a.logit_x = reinterpret_cast<unsigned long long *>(ws + wl.logit_off);
    a.logit_stride = DEC_RING * wl.n_logit;
    a.h_x = reinterpret_cast<unsigned long long *>(ws + wl.h_off);
    a.y_x = a.h_x + wl.n_h;
    a.word_stride = DEC_RING * wl.n_h;
    a.spin_limit = d.spin_limit_ticks;

    // both regions are contiguous from logit_off to the end of the workspace
    hipLaunchKernelGGL(decode_chain_clear, dim3(1), dim3(1024), 0, stream, a.abort_flag, a.logit_x,
                       (int)((wl.total - wl.logit_off) / sizeof(unsigned long long)));
    void *params[] = {&a};
    const void *fn = nullptr;
    const bool few = KI <= 4 * 512;                  // down-row chunks per lane: 4 or 12
    switch (d.H / 512) {
    case 1: fn = few ? reinterpret_cast<const void *>(decode_chain_kernel<1, 4, 1>) : reinterpret_cast<const void *>(decode_chain_kernel<1, 12, 1>); break;
    case 2: fn = few ? reinterpret_cast<const void *>(decode_chain_kernel<2, 4, 1>) : reinterpret_cast<const void *>(decode_chain_kernel<2, 12, 1>); break;
    case 4: fn = few ? reinterpret_cast<const void *>(decode_chain_kernel<4, 4, 1>) : reinterpret_cast<const void *>(decode_chain_kernel<4, 12, 1>); break;
    case 8: fn = few ? reinterpret_cast<const void *>(decode_chain_kernel<8, 4, 2>) : reinterpret_cast<const void *>(decode_chain_kernel<8, 12, 2>); break;
    default: return fail(REMOE_E_UNSUPPORTED, "decode supports hidden in {512, 1024, 2048, 4096} (got %d)", d.H);
    }
    // Every workgroup must be resident (the exchanges wait for all of them).  An ordinary launch of one
    // workgroup per compute unit gives that once the occupancy query confirms a workgroup fits; should
    // other work hold compute units for long, the bounded waits end the kernel with the abort word set
    // instead of hanging.  (A cooperative launch would check the same, but kernel tracing tools on this
    // software stack crash at process exit after one.)  Unused dynamic LDS lifts the workgroup above
    // half a compute unit's 160 KB, so that no two workgroups share a compute unit while another idles.
    hipFuncAttributes attr;
    REMOE_HIP_TRY(hipFuncGetAttributes(&attr, fn));
    const size_t half_lds = 80 * 1024 + 256;
    const size_t pad = attr.sharedSizeBytes < half_lds ? half_lds - attr.sharedSizeBytes : 0;
    int per_cu = 0;
    REMOE_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, CH_THREADS, pad));
    if (per_cu < 1) return fail(REMOE_E_UNSUPPORTED, "decode: a workgroup does not fit one compute unit");
    REMOE_HIP_TRY(hipLaunchKernel(fn, dim3(G), dim3(CH_THREADS), params, pad, stream));
    return REMOE_OK;
}

}  // namespace remoe
