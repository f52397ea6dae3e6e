// M = 1 decode: the whole MoE layer for one token per step, weights streamed once from HBM.
//
// At one token per step the layer (Sec. 3.1 routing, Sec. 4.1 step 5 expert execution) is a chain
// of matrix-vector products with about one flop per byte, so the matrix cores are useless and the
// only roofline is HBM bandwidth: per layer-step the fp32 router matrix (N_r x H) and the three
// matrices of the K selected experts are read exactly once.  One persistent kernel runs all layers
// of all steps of a call: one workgroup of 8 wavefronts per compute unit, three phases per
// layer-step separated by grid-wide barriers (an atomic counter in device memory):
//   1. router   : every wavefront dots one 256-wide segment of one router row with x; partial
//                 logits go to device memory;                                       -- barrier --
//      top-k    : wavefront 0 of every workgroup sums the partials and runs the wavefront-shuffle
//                 top-k / softmax (identical result everywhere, so no broadcast is needed);
//   2. gate/up  : the K*I SwiGLU activations are dealt out in contiguous runs, each wavefront
//                 streams the gate and up rows of its activations with 16-byte coalesced loads;
//                 h goes to device memory in fp32;                                  -- barrier --
//   3. down     : every wavefront owns output rows; for each it streams the K down-projection rows
//                 (already prefetched into registers before the barrier, since the experts are
//                 known) against h staged in LDS, weighted by the gate weights.     -- barrier --
// Layers run strictly in order, as a real decoder would.  The routing-trace statistics the paper
// optimises are updated online in the same kernel (one wavefront, right after the top-k): the
// adjacent-step overlap |E_t ∩ E_{t-1}| (Eq. 1) and the LRU misses |E_t \ C_t| (App. E.2) for up to
// four cache capacities at once, from one per-expert "last used" table per layer.
//
// Every wait is bounded: a workgroup that waits longer than the limit raises an abort flag, every
// other workgroup sees the flag at its next wait, and the whole grid drains.
#include "common.h"
#include "decode_common.h"
#include "topk.h"

namespace remoe {

namespace {

constexpr int DC_THREADS = DEC_THREADS;
constexpr int DC_WAVES = DC_THREADS / 64;
constexpr int DC_SEG = DEC_SEG;
constexpr int DC_MAX_KI = 6144;      // K * I floats of h staged in LDS (24 KB)
constexpr int DC_MAX_CAPS = DEC_MAX_CAPS;
constexpr int DC_MAX_GRID = DEC_MAX_GRID;
constexpr int DC_MAX_LAYERS = DEC_MAX_LAYERS;
constexpr int DC_MAX_DCH = 12;       // down-projection chunks per lane per output row (K * I <= 6144)

struct DecodeArgs {
    const void *const *layers;   // [L][4] device pointers: w_router, w_gate, w_up, w_down
    const bf16_t *x;             // [T_total, H]
    int64_t steps_total, step0, n_steps;
    int n_layers, H, N, I, K, renorm;
    bf16_t *y;                   // [T_total, L, H]
    int32_t *out_idx;            // [L, T_total, K]
    float *out_w;                // [L, T_total, K]
    int n_caps;
    int caps[DC_MAX_CAPS];
    unsigned long long expert_bytes;
    uint32_t *lru_state;         // [L, N] last use (global step + 1), 0 = never
    uint8_t *out_overlap;        // [L, T_total]
    uint8_t *out_miss;           // [n_caps, L, T_total]
    unsigned long long *sum_overlap;   // [L]
    unsigned long long *total_miss;    // [n_caps, L]
    unsigned long long *bytes_fetched; // [n_caps, L]
    unsigned long long *logit_part;   // [N * H / DC_SEG] (phase tag << 32) | float bits
    float *hbuf;                 // [K * I]
    uint32_t *bar;               // grid barrier flags, one per workgroup, zero at launch
    uint32_t *abort_flag;        // zero at launch
    unsigned long long spin_limit;   // wall-clock ticks (100 MHz) a single wait may last
};

template <int XCH>
__global__ __launch_bounds__(DC_THREADS) void decode_kernel(const DecodeArgs a)
{
    __shared__ float hl[DC_MAX_KI];
    __shared__ float lz[128];      // logits of the current layer-step
    __shared__ float lpart[128 * 16];   // their per-segment partial sums (H <= 4096)
    __shared__ int rank_part[DC_WAVES][128];
    __shared__ int sel_e[8];
    __shared__ float sel_w[8];
    __shared__ float sel_z[9];
    __shared__ int bar_ok;
    __shared__ TraceLds ts;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int G = gridDim.x;
    const int W = G * DC_WAVES;                 // wavefronts in the grid
    const int gw = blockIdx.x * DC_WAVES + wave;  // this wavefront's global index
    const int H = a.H, N = a.N, I = a.I, K = a.K;
    const int segs = H / DC_SEG;
    const int KI = K * I;
    const int items_per_wave = (KI + W - 1) / W;
    const int rows_per_wave = (H + W - 1) / W;
    const int dchunks = KI / 8;                 // 16-byte chunks of one output row's K down rows
    const int chunks_per_row = I / 8;
    const bool stats_wave = blockIdx.x == G - 1 && wave == DC_WAVES - 1;
    const int n_items1 = N * segs;              // router work items: (expert, 256-wide segment)
    uint32_t phase = 0;

    if (blockIdx.x == G - 1) {                  // trace state -> LDS
        for (int q = tid; q < a.n_layers * 128; q += DC_THREADS) {
            const int l = q >> 7, e = q & 127;
            ts.last[l][e] = (e < N) ? a.lru_state[l * N + e] : 0u;
        }
        for (int q = tid; q < a.n_layers; q += DC_THREADS) {
            ts.sum_ov[q] = a.sum_overlap[q];
            for (int c = 0; c < a.n_caps; ++c) ts.tot[c][q] = a.total_miss[c * a.n_layers + q];
        }
    }
    __syncthreads();

    // the router row segment of this wavefront's first work item of the NEXT layer is fetched ahead
    floatx4_t wr_pf = {0.f, 0.f, 0.f, 0.f};
    const int e1 = gw / segs, k1 = (gw - e1 * segs) * DC_SEG + lane * 4;
    if (gw < n_items1)
        wr_pf = load_global<floatx4_t>(static_cast<const float *>(table_ptr(a.layers, 0)) + (int64_t)e1 * H + k1);

#pragma unroll 1
    for (int64_t s = 0; s < a.n_steps; ++s) {
        const int64_t g = a.step0 + s;
        const bf16_t *xg = a.x + g * H;
#pragma unroll 1
        for (int layer = 0; layer < a.n_layers; ++layer) {
            const float *w_router = static_cast<const float *>(table_ptr(a.layers, layer * 4 + 0));
            const bf16_t *w_gate = static_cast<const bf16_t *>(table_ptr(a.layers, layer * 4 + 1));
            const bf16_t *w_up = static_cast<const bf16_t *>(table_ptr(a.layers, layer * 4 + 2));
            const bf16_t *w_down = static_cast<const bf16_t *>(table_ptr(a.layers, layer * 4 + 3));

            // ---- phase 1: partial router logits --------------------------------------------------
#pragma unroll 1
            for (int item = gw; item < n_items1; item += W) {
                const int e = item / segs, sg = item - e * segs;
                const int k0 = sg * DC_SEG + lane * 4;
                floatx4_t wv = wr_pf;
                if (item != gw) wv = load_global<floatx4_t>(w_router + (int64_t)e * H + k0);
                const uint2 xb = *reinterpret_cast<const uint2 *>(xg + k0);
                float p = wv.x * __uint_as_float(xb.x << 16);
                p = fmaf(wv.y, __uint_as_float(xb.x & 0xFFFF0000u), p);
                p = fmaf(wv.z, __uint_as_float(xb.y << 16), p);
                p = fmaf(wv.w, __uint_as_float(xb.y & 0xFFFF0000u), p);
                p = wave_sum(p);
                if (lane == 0) put_tagged(&a.logit_part[item], p, phase + 1);
            }
            // this lane's share of x, widened once per layer-step: chunk c covers k = (c*64 + lane)*8 ..
            float xr[XCH][8];
#pragma unroll
            for (int c = 0; c < XCH; ++c) {
                const u32x4_t xb = *reinterpret_cast<const u32x4_t *>(xg + (c * 64 + lane) * 8);
                xr[c][0] = __uint_as_float(xb.x << 16); xr[c][1] = __uint_as_float(xb.x & 0xFFFF0000u);
                xr[c][2] = __uint_as_float(xb.y << 16); xr[c][3] = __uint_as_float(xb.y & 0xFFFF0000u);
                xr[c][4] = __uint_as_float(xb.z << 16); xr[c][5] = __uint_as_float(xb.z & 0xFFFF0000u);
                xr[c][6] = __uint_as_float(xb.w << 16); xr[c][7] = __uint_as_float(xb.w & 0xFFFF0000u);
            }
            // ---- first grid-wide rendezvous: the partial logits carry the phase number as a tag, so
            // polling for them IS the barrier (one memory round trip once the last one is written) ------
            ++phase;
            if (!gather_tagged(a, lpart, n_items1, phase, &bar_ok)) return;

            // ---- top-k and softmax by rank counting (every workgroup, same result everywhere) -------
            // Every wavefront sums all N logits (cheap) and counts, for its 1/8 of the experts q, how many
            // beat expert e (larger logit, or equal logit and lower id); ranks 0..K-1 are the selection,
            // already in descending-logit order.
            {
                const float NEG_INF = -__builtin_inff();
                float v0 = NEG_INF, v1 = NEG_INF;
                if (lane < N) {
                    v0 = 0.f;
                    for (int q = 0; q < segs; ++q) v0 += lpart[lane * segs + q];
                }
                if (lane + 64 < N) {
                    v1 = 0.f;
                    for (int q = 0; q < segs; ++q) v1 += lpart[(lane + 64) * segs + q];
                }
                if (wave == 0) { lz[lane] = v0; lz[lane + 64] = v1; }
                // this wavefront compares against experts q = wave, wave + 8, ...; the logit of q sits in
                // lane q & 63 (v0 or v1), so it is fetched with a lane read instead of LDS
                int r0 = 0, r1 = 0;
                for (int q = wave; q < N; q += DC_WAVES) {
                    const float zq = __shfl((q < 64) ? v0 : v1, q & 63, 64);
                    r0 += (zq > v0) || (zq == v0 && q < lane);
                    r1 += (zq > v1) || (zq == v1 && q < lane + 64);
                }
                rank_part[wave][lane] = r0;
                rank_part[wave][lane + 64] = r1;
            }
            __syncthreads();
            if (wave == 0) {
                const float v0 = lz[lane], v1 = lz[lane + 64];
                int r0 = 0, r1 = 0;
#pragma unroll
                for (int w = 0; w < DC_WAVES; ++w) { r0 += rank_part[w][lane]; r1 += rank_part[w][lane + 64]; }
                if (lane < N && r0 <= K) { sel_z[r0] = v0; if (r0 < K) sel_e[r0] = lane; }
                if (lane + 64 < N && r1 <= K) { sel_z[r1] = v1; if (r1 < K) sel_e[r1] = lane + 64; }
                const float zmax = sel_z[0];
                const float den = wave_sum(((lane < N) ? expf(v0 - zmax) : 0.f) + ((lane + 64 < N) ? expf(v1 - zmax) : 0.f));
                const float my_p = (lane < K) ? expf(sel_z[lane] - zmax) : 0.f;
                float wgt = my_p / den;
                if (a.renorm) wgt = my_p / wave_sum(my_p);
                if (lane < K) {
                    sel_w[lane] = wgt;
                    if (blockIdx.x == 0) {
                        const int64_t o = ((int64_t)layer * a.steps_total + g) * K + lane;
                        a.out_idx[o] = sel_e[lane];
                        a.out_w[o] = wgt;
                    }
                }
            }
            __syncthreads();

            // ---- phase 2: gate / up rows of the selected experts, SwiGLU -----------------------------
            // Row bases are wave-uniform (scalar registers); a lane adds its own 32-bit offset.  Two
            // register sets roll over the wavefront's activations (the loads of the next one or two are
            // in flight while one is reduced), and the down-projection rows of phase 3 are requested
            // right behind the last of them, so HBM keeps streaming across the coming barrier.
            u32x4_t dv[DC_MAX_DCH];
            const int row_first = gw * rows_per_wave;
            const char *wd_bytes = reinterpret_cast<const char *>(w_down);
#define DC_ISSUE_DOWN()                                                                              \
    _Pragma("unroll") for (int c = 0; c < DC_MAX_DCH; ++c) {                                          \
        const int q_ = c * 64 + lane;                                                                \
        if (q_ < dchunks && row_first < H) {                                                         \
            const int j_ = q_ / chunks_per_row, pos_ = (q_ - j_ * chunks_per_row) * 8;               \
            const uint32_t off_ = (uint32_t)((((int64_t)sel_e[j_] * H + row_first) * I + pos_) * 2); \
            dv[c] = load_global_stream<u32x4_t>(wd_bytes + off_);                             \
        }                                                                                            \
    }
            {
                const int item0 = gw * items_per_wave;
                int nit = KI - item0;
                if (nit > items_per_wave) nit = items_per_wave;
                const int loff = lane * 8;
                u32x4_t gA[XCH], uA[XCH], gB[XCH], uB[XCH];
#define DC_LOAD_ITEM(gv, uv, it)                                                                     \
    {                                                                                                \
        const int item_ = item0 + (it);                                                              \
        const int j_ = item_ / I, i_ = item_ - j_ * I;                                               \
        const int e_ = __builtin_amdgcn_readfirstlane(sel_e[j_]);                                    \
        const bf16_t *gp_ = w_gate + ((int64_t)e_ * I + i_) * H;                                     \
        const bf16_t *up_ = w_up + ((int64_t)e_ * I + i_) * H;                                       \
        _Pragma("unroll") for (int c = 0; c < XCH; ++c) {                                             \
            gv[c] = load_global_stream<u32x4_t>(gp_ + loff + c * 512);                        \
            uv[c] = load_global_stream<u32x4_t>(up_ + loff + c * 512);                        \
        }                                                                                            \
    }
#define DC_REDUCE_ITEM(gv, uv, it)                                                                   \
    {                                                                                                \
        float gs_ = 0.f, us_ = 0.f;                                                                  \
        _Pragma("unroll") for (int c = 0; c < XCH; ++c) {                                             \
            gs_ = dot8(gv[c], xr[c], gs_);                                                           \
            us_ = dot8(uv[c], xr[c], us_);                                                           \
        }                                                                                            \
        gs_ = wave_sum(gs_);                                                                         \
        us_ = wave_sum(us_);                                                                         \
        if (lane == 0) put_shared(&a.hbuf[item0 + (it)], gs_ / (1.0f + expf(-gs_)) * us_);           \
    }
                bool down_issued = false;
                if (nit > 0) DC_LOAD_ITEM(gA, uA, 0)
                if (nit > 1) DC_LOAD_ITEM(gB, uB, 1)
                if (nit <= 2) { DC_ISSUE_DOWN() down_issued = true; }
                // the statistics ride on the latency of the loads just issued
                if (stats_wave) online_trace_stats(a, ts, layer, g, sel_e, lane);
#pragma unroll 1
                for (int it = 0; it < nit; it += 2) {
                    DC_REDUCE_ITEM(gA, uA, it)
                    if (it + 2 < nit) DC_LOAD_ITEM(gA, uA, it + 2)
                    if (!down_issued && it + 3 >= nit) { DC_ISSUE_DOWN() down_issued = true; }
                    if (it + 1 < nit) {
                        DC_REDUCE_ITEM(gB, uB, it + 1)
                        if (it + 3 < nit) DC_LOAD_ITEM(gB, uB, it + 3)
                    }
                }
            }
            if (!grid_barrier(a, ++phase, &bar_ok)) return;

            // ---- phase 3: down projection; h is staged in LDS already multiplied by the gate weight ----
            for (int q0 = tid; q0 < KI; q0 += DC_THREADS * 4) {
                float hv[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {          // four loads in flight per thread
                    const int q = q0 + u * DC_THREADS;
                    hv[u] = (q < KI) ? get_shared(&a.hbuf[q]) : 0.f;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int q = q0 + u * DC_THREADS;
                    if (q < KI) hl[q] = hv[u] * sel_w[q / I];
                }
            }
            // router row segment of the next layer-step, in flight across the last barrier
            {
                int nl = layer + 1;
                if (nl == a.n_layers) nl = 0;
                if (gw < n_items1)
                    wr_pf = load_global<floatx4_t>(static_cast<const float *>(table_ptr(a.layers, nl * 4)) + (int64_t)e1 * H + k1);
            }
            __syncthreads();
#pragma unroll 1
            for (int rw = 0; rw < rows_per_wave; ++rw) {
                const int o = row_first + rw;
                if (o >= H) break;
                float acc = 0.f;
#pragma unroll
                for (int c = 0; c < DC_MAX_DCH; ++c) {
                    const int q = c * 64 + lane;
                    if (q < dchunks) {
                        u32x4_t wv = dv[c];
                        if (rw > 0) {   // further rows of this wavefront are fetched on the spot
                            const int j = q / chunks_per_row, pos = (q - j * chunks_per_row) * 8;
                            const uint32_t off = (uint32_t)((((int64_t)sel_e[j] * H + o) * I + pos) * 2);
                            wv = load_global_stream<u32x4_t>(wd_bytes + off);
                        }
                        acc = dot8(wv, &hl[q * 8], acc);
                    }
                }
                acc = wave_sum(acc);
                if (lane == 0) a.y[(g * a.n_layers + layer) * H + o] = f32_to_bf16(acc);
            }
            if (!grid_barrier(a, ++phase, &bar_ok)) return;
        }
    }

    if (blockIdx.x == G - 1) {                  // trace state back to device memory
        __syncthreads();
        for (int q = tid; q < a.n_layers * 128; q += DC_THREADS) {
            const int l = q >> 7, e = q & 127;
            if (e < N) a.lru_state[l * N + e] = ts.last[l][e];
        }
        for (int q = tid; q < a.n_layers; q += DC_THREADS) {
            a.sum_overlap[q] = ts.sum_ov[q];
            for (int c = 0; c < a.n_caps; ++c) {
                a.total_miss[c * a.n_layers + q] = ts.tot[c][q];
                a.bytes_fetched[c * a.n_layers + q] = ts.tot[c][q] * a.expert_bytes;
            }
        }
    }
}

__global__ void decode_clear_flags(uint32_t *bar, int n, uint32_t *abort_flag, unsigned long long *tagged, int n_tagged)
{
    for (int q = threadIdx.x; q < n; q += blockDim.x) bar[q] = 0u;
    for (int q = threadIdx.x; q < n_tagged; q += blockDim.x) tagged[q] = 0ull;   // tag 0 = no phase
    if (threadIdx.x == 0) *abort_flag = 0u;
}

}  // namespace

size_t decode_workspace_bytes(int H, int N, int I, int K) { return decode_ws_layout(H, N, I, K).total; }

remoe_status launch_decode(const DecodeLaunch &d, hipStream_t stream)
{
    if (d.H != 512 && d.H != 1024 && d.H != 2048 && d.H != 4096)
        return fail(REMOE_E_UNSUPPORTED, "decode supports hidden in {512, 1024, 2048, 4096} (got %d)", d.H);
    if (d.I % 8 != 0 || d.K * d.I > DC_MAX_KI)
        return fail(REMOE_E_UNSUPPORTED, "decode needs inter %% 8 == 0 and top_k * inter <= %d", DC_MAX_KI);
    if (d.n_layers > DC_MAX_LAYERS)
        return fail(REMOE_E_UNSUPPORTED, "decode keeps the trace state of at most %d layers (got %d)", DC_MAX_LAYERS, d.n_layers);
    if (d.n_caps < 0 || d.n_caps > DC_MAX_CAPS)
        return fail(REMOE_E_INVALID_ARG, "n_caps %d outside 0..%d", d.n_caps, DC_MAX_CAPS);
    int dev = 0, n_cu = 0;
    REMOE_HIP_TRY(hipGetDevice(&dev));
    REMOE_HIP_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
    if (n_cu < 1) return fail(REMOE_E_HIP, "device reports no compute units");
    // one workgroup per compute unit, all resident at once (checked against the occupancy below)
    const int G = n_cu;
    const int W = G * DC_WAVES;
    if ((d.K * d.I / 8 + 63) / 64 > DC_MAX_DCH)
        return fail(REMOE_E_UNSUPPORTED, "decode: top_k * inter too large for the register prefetch");
    (void)W;

    DecodeArgs a;
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
    for (int c = 0; c < DC_MAX_CAPS; ++c) a.caps[c] = (c < d.n_caps) ? d.caps[c] : 0;
    a.expert_bytes = d.expert_bytes;
    a.lru_state = d.lru_state;
    a.out_overlap = d.out_overlap;
    a.out_miss = d.out_miss;
    a.sum_overlap = reinterpret_cast<unsigned long long *>(d.sum_overlap);
    a.total_miss = reinterpret_cast<unsigned long long *>(d.total_miss);
    a.bytes_fetched = reinterpret_cast<unsigned long long *>(d.bytes_fetched);
    char *ws = static_cast<char *>(d.workspace);
    if (G > DC_MAX_GRID) return fail(REMOE_E_UNSUPPORTED, "decode: %d compute units exceed the barrier's %d flags", G, DC_MAX_GRID);
    a.abort_flag = reinterpret_cast<uint32_t *>(ws + 128);
    a.bar = reinterpret_cast<uint32_t *>(ws + 256);
    const DecodeWsLayout wl = decode_ws_layout(d.H, d.N, d.I, d.K);
    a.logit_part = reinterpret_cast<unsigned long long *>(ws + wl.logit_off);
    a.hbuf = reinterpret_cast<float *>(ws + wl.h_off);
    a.spin_limit = d.spin_limit_ticks;

    hipLaunchKernelGGL(decode_clear_flags, dim3(1), dim3(256), 0, stream, a.bar, G, a.abort_flag, a.logit_part,
                       d.N * (d.H / DC_SEG));
    void *params[] = {&a};
    const void *fn = nullptr;
    switch (d.H / 512) {
    case 1: fn = reinterpret_cast<const void *>(decode_kernel<1>); break;
    case 2: fn = reinterpret_cast<const void *>(decode_kernel<2>); break;
    case 4: fn = reinterpret_cast<const void *>(decode_kernel<4>); break;
    case 8: fn = reinterpret_cast<const void *>(decode_kernel<8>); break;
    default: return fail(REMOE_E_UNSUPPORTED, "decode supports hidden in {512, 1024, 2048, 4096} (got %d)", d.H);
    }
    // The grid barrier needs every workgroup resident.  An ordinary launch of one workgroup per
    // compute unit gives that once the occupancy query confirms a workgroup fits; should other work
    // hold compute units for long, the bounded waits end the kernel with the abort word set instead
    // of hanging.  (A cooperative launch would check the same, but kernel tracing tools on this
    // software stack crash at process exit after one.)
    // Unused dynamic LDS lifts the workgroup above half a compute unit's 160 KB, so that no two
    // workgroups share a compute unit while another one idles.
    hipFuncAttributes attr;
    REMOE_HIP_TRY(hipFuncGetAttributes(&attr, fn));
    const size_t half_lds = 80 * 1024 + 256;
    const size_t pad = attr.sharedSizeBytes < half_lds ? half_lds - attr.sharedSizeBytes : 0;
    int per_cu = 0;
    REMOE_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, DC_THREADS, pad));
    if (per_cu < 1) return fail(REMOE_E_UNSUPPORTED, "decode: a workgroup does not fit one compute unit");
    REMOE_HIP_TRY(hipLaunchKernel(fn, dim3(G), dim3(DC_THREADS), params, pad, stream));
    return REMOE_OK;
}

}  // namespace remoe
