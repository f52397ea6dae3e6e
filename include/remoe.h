/*
 * remoe.h — C ABI of the MI355X (gfx950) MoE-layer hot path and routing-trace statistics.
 *
 * Notation follows the paper's preliminaries (Sec. 3.1): N_r routed experts, router parameters
 * theta_gate, hidden state h_t, routing distribution P_t, selected set E_t with |E_t| = K,
 * per-layer expert-cache capacity C.  In this header: T = tokens in a call, H = hidden size,
 * I = routed expert intermediate size, I_s = total shared-expert intermediate size.
 *
 * General conventions
 *   - Every pointer is a DEVICE pointer owned by the caller unless marked "host".  The library
 *     never allocates, frees or keeps caller-visible memory; scratch comes from the caller's
 *     workspace (remoe_workspace_bytes).
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the null stream) and the
 *     host is never synchronised; outputs are valid once the stream reaches the end of the call.
 *   - Matrices are row-major [out_features, in_features] (reduction dimension contiguous).
 *   - Expert ids are 0-based (the paper counts from 1).
 *   - Every entry point validates its arguments before launching anything and returns a negative
 *     remoe_status on error; remoe_last_error() then holds a message.  No exception crosses the ABI.
 *   - Expert ids inside a trace handed to trace_reuse / lru_simulate must lie in [0, n_experts);
 *     ids outside are ignored by the kernels (they never index memory with them).
 */
#ifndef REMOE_H
#define REMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    REMOE_OK = 0,
    REMOE_E_INVALID_ARG = -1,
    REMOE_E_UNSUPPORTED = -2,
    REMOE_E_WORKSPACE = -3,
    REMOE_E_HIP = -4
} remoe_status;

typedef enum { REMOE_F32 = 0, REMOE_BF16 = 1 } remoe_dtype;

/* Shape of one MoE layer. */
typedef struct {
    int32_t hidden;        /* H; multiple of 32 (of 128 when dtype is bf16)                         */
    int32_t n_experts;     /* N_r, 1..128                                                            */
    int32_t inter;         /* I; multiple of 64 when dtype is bf16                                   */
    int32_t top_k;         /* K, 1..min(N_r, 8)                                                      */
    int32_t renorm;        /* 0: w = P_t[E_t]; 1: w divided by the sum over the K selected           */
    int32_t shared_inter;  /* I_s, 0 = no shared expert; multiple of 64 when dtype is bf16           */
    int32_t shared_gate;   /* 1: shared expert output scaled by sigmoid(ws_scale . x)                */
    int32_t dtype;         /* remoe_dtype of x, expert weights and y; the router is always fp32      */
} remoe_layer_desc;

/* Library version (major * 10000 + minor * 100 + patch). Host call, no GPU work. */
int32_t remoe_version(void);

/* Message of the calling thread's last failed call (static thread-local storage, never NULL). */
const char *remoe_last_error(void);

/* Bytes of workspace moe_forward needs for `n_tokens` tokens of this layer shape (0 on invalid
 * arguments, with remoe_last_error set).  Host call, no GPU work. */
size_t remoe_workspace_bytes(const remoe_layer_desc *desc, int64_t n_tokens);

/*
 * moe_route — the router of Sec. 3.1: P_t = Softmax(h_t^T theta_gate), E_t = Top-K(P_t).
 *
 *   x          [T, H]    hidden states, desc->dtype (bf16 values are widened exactly to fp32)
 *   w_router   [N_r, H]  fp32 gate matrix, no bias
 *   out_idx    [T, K]    int32 expert ids, ordered by descending logit, ties to the lower id
 *   out_w      [T, K]    fp32 gate weights P_t[E_t] (softmax over all N_r experts), divided by
 *                        their sum when desc->renorm
 *   out_margin [T]       fp32 logit_(K) - logit_(K+1) (+inf when K == N_r), or NULL
 *   out_probs  [T, N_r]  fp32 P_t, or NULL
 *
 * The logits carry fp32 accuracy.  fp32 hidden states are multiplied on the fp32 matrix cores.
 * bf16 hidden states are multiplied on the bf16 matrix cores against the gate matrix split into
 * three bf16 pieces per weight (hi + mid + lo, 24 significand bits in all), so every product is
 * exact in fp32 and the sums are fp32.  T may be 0 (nothing is launched).
 * Only hidden, n_experts, top_k, renorm and dtype of `desc` are read.
 */
remoe_status moe_route(const remoe_layer_desc *desc, const void *x, int64_t n_tokens,
                       const float *w_router, int32_t *out_idx, float *out_w,
                       float *out_margin, float *out_probs, void *stream);

/*
 * moe_forward — one fine-grained MoE layer (Sec. 3.1 routing; Sec. 4.1 step 5: the selected
 * Top-K experts execute as in the base model; shared experts always execute and lie outside P_t):
 *
 *   y[t] = sum_{j<K} out_w[t,j] * FFN_{out_idx[t,j]}(x[t])  +  s_t * FFN_shared(x[t])
 *   FFN_e(x) = W_down[e] ( silu(W_gate[e] x) * (W_up[e] x) ),  silu(z) = z / (1 + exp(-z))
 *   s_t = sigmoid(ws_scale . x[t]) when desc->shared_gate, else 1
 *
 *   x        [T, H]          desc->dtype
 *   w_router [N_r, H]        fp32
 *   w_gate   [N_r, I, H]     desc->dtype        w_up [N_r, I, H]      w_down [N_r, H, I]
 *   ws_gate  [I_s, H]        desc->dtype        ws_up [I_s, H]        ws_down [H, I_s]
 *                            (NULL when shared_inter == 0)
 *   ws_scale [H]             fp32 (NULL unless shared_gate)
 *   y        [T, H]          desc->dtype
 *   out_idx  [T, K] int32,   out_w [T, K] fp32  — the routing, as moe_route returns it
 *   workspace                at least remoe_workspace_bytes(desc, T) bytes, 256-byte aligned;
 *                            contents are scratch and meaningless afterwards
 *
 * No residual connection and no normalisation.  bf16 layers multiply on the bf16 matrix cores
 * with fp32 accumulation; the SwiGLU activations and the per-(token, expert) outputs are stored
 * in bf16 between kernels and the K (+1) rows of a token are summed in fp32.  fp32 layers
 * compute in fp32 throughout.  The result is deterministic (no floating-point atomics).
 */
remoe_status moe_forward(const remoe_layer_desc *desc, const void *x, int64_t n_tokens,
                         const float *w_router,
                         const void *w_gate, const void *w_up, const void *w_down,
                         const void *ws_gate, const void *ws_up, const void *ws_down,
                         const float *ws_scale,
                         void *y, int32_t *out_idx, float *out_w,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * trace_reuse — adjacent-step expert overlap, the numerator of IR_t in Eq. 1 (Sec. 3.2):
 *
 *   out_overlap[s, 0] = 0,  out_overlap[s, t] = |E_t ∩ E_{t-1}|  (sets of distinct ids)
 *   out_sum[s]        = sum_t out_overlap[s, t]     (EOR = out_sum / (K (T-1)), left to the caller)
 *
 *   idx         [S, T, K]  int32 routing trace; S independent traces, one per (sequence, layer)
 *   out_overlap [S, T]     uint8
 *   out_sum     [S]        uint64
 *
 * Traces never see each other.  n_experts <= 128, top_k <= 64.  S or T may be 0.
 */
remoe_status trace_reuse(const int32_t *idx, int64_t n_seq, int64_t n_steps,
                         int32_t top_k, int32_t n_experts,
                         uint8_t *out_overlap, uint64_t *out_sum, void *stream);

/*
 * lru_simulate — per-layer LRU expert cache of capacity C (Sec. 5.1 "Expert-cache simulation",
 * App. A cache model, App. E.2 unique-miss accounting):
 *
 *   out_miss[s, t]    = |U_t \ C_t|, U_t the distinct ids of step t, C_t the resident set BEFORE
 *                       the step is served
 *   out_total_miss[s] = sum_t out_miss[s, t]                         (#uMiss)
 *   out_bytes[s]      = out_total_miss[s] * expert_bytes             (bytes fetched)
 *
 * After counting, the step's experts become the most recent ones (within a step in ascending id
 * order) and the cache keeps the C most recent distinct experts.
 *
 *   state [S, N_r] uint32, or NULL.  Entry e holds (global step of e's last use) + 1, 0 = never
 *         used.  NULL: every trace starts cold and the final state is discarded.  Non-NULL: the
 *         state is read, updated and written back, so a trace can be fed in pieces (online decode:
 *         n_steps = 1 per call); a zero-filled state is a cold cache.  Pieces are fed in order: step0 is
 *         larger than every step the state already records.
 *   step0 global index of the first step of this call (>= 0; step0 + n_steps must stay below
 *         2^24 so that recency keys fit 32 bits).
 *
 * n_experts <= 128, top_k <= 64, capacity >= 1.  S or T may be 0.
 */
remoe_status lru_simulate(const int32_t *idx, int64_t n_seq, int64_t n_steps,
                          int32_t top_k, int32_t n_experts, int32_t capacity,
                          uint64_t expert_bytes, int64_t step0, uint32_t *state,
                          uint8_t *out_miss, uint64_t *out_total_miss, uint64_t *out_bytes,
                          void *stream);

/*
 * moe_decode — M = 1 decode: the MoE layer of every one of `n_layers` layers for `n_steps`
 * consecutive single-token steps, as one persistent kernel bound by HBM bandwidth (the B = 1
 * regime of Sec. 3: per layer-step the router matrix and the K selected experts' weights are read
 * once), with the routing-trace statistics updated online after every step (adjacent overlap,
 * Eq. 1; LRU misses of App. E.2 for up to 4 capacities at once).  Steps run strictly in order.
 *
 *   layer_order     how the layers of one step are scheduled.  Every layer of a step reads the same
 *                   input row x[g] (this path has no attention or residual between MoE layers), so the
 *                   layers of a step do not depend on each other and both orders give the same result:
 *                   REMOE_DECODE_CHAINED    a layer starts only after the previous layer has finished
 *                                           on every compute unit, as in a decoder whose layers feed
 *                                           each other.  Per layer-step the grid exchanges three sets
 *                                           of values (router logits, the K * I activations, the H
 *                                           output values) as tagged words that every workgroup
 *                                           publishes and a dedicated wavefront per workgroup collects;
 *                                           there is no grid-wide barrier.  With W = 8 * compute
 *                                           units it needs ceil(top_k * inter / W) <= 3,
 *                                           ceil(hidden / W) <= 1 (<= 2 for hidden = 4096) and
 *                                           n_experts * hidden / 256 <= W; other shapes are refused
 *                                           with REMOE_E_UNSUPPORTED;
 *                   REMOE_DECODE_PIPELINED  the layers of a step overlap.  The compute units are split
 *                                           into 8 groups (one per XCD); group x owns layers x, x + 8,
 *                                           ... and runs them as a software pipeline: while one of its
 *                                           layers' gate/up rows stream, the next layers' router logits
 *                                           and top-k are computed and an earlier layer's down rows are
 *                                           read, so no wait sits between two HBM streams.  With
 *                                           W = 8 * compute units / groups wavefronts per group (256
 *                                           on MI355X; a device whose compute-unit count is not a
 *                                           multiple of 8 runs as a single group) it needs
 *                                           n_experts * hidden / 256 <= min(2048, 4 W) and
 *                                           W * ceil(ceil(top_k * inter / W) / 3) <= 2048;
 *                                           other shapes are refused with REMOE_E_UNSUPPORTED.
 *
 *   desc            bf16 layers without shared expert; hidden in {512, 1024, 2048, 4096},
 *                   inter % 64 == 0 (as for every bf16 layer), top_k * inter <= 6144
 *   layer_weights   DEVICE array [n_layers][4] of device pointers: w_router [N_r,H] fp32,
 *                   w_gate [N_r,I,H], w_up [N_r,I,H], w_down [N_r,H,I] (bf16)
 *   x               [steps_total, H] bf16; step g reads row g (every layer sees the same row)
 *   step0, n_steps  the steps [step0, step0 + n_steps) of the run are executed by this call
 *   y               [steps_total, n_layers, H] bf16, rows of the executed steps are written
 *   out_idx, out_w  [n_layers, steps_total, K] int32 / fp32: the routing of every layer-step
 *   capacities      HOST array [n_caps] of LRU capacities (n_caps 0..4)
 *   lru_state       [n_layers, N_r] uint32, (step of last use) + 1, 0 = never; zero = cold cache;
 *                   read and updated, so a run can be split over several calls
 *   out_overlap     [n_layers, steps_total] uint8;  out_miss [n_caps, n_layers, steps_total] uint8
 *   sum_overlap     [n_layers] uint64;  total_miss, bytes_fetched [n_caps, n_layers] uint64:
 *                   running sums, ADDED to by every call (zero them before the first)
 *   workspace       remoe_decode_workspace_bytes(desc) bytes, 256-byte aligned.  The 32-bit word at
 *                   byte 128 is an abort flag: non-zero after the
 *                   call has completed means a wait inside the kernel exceeded `spin_limit_us` and
 *                   the outputs of this call are invalid (every workgroup still exits).
 *   spin_limit_us   upper bound of a single wait for other workgroups' values in microseconds (0 = 2 seconds)
 *
 * The kernel is persistent: one workgroup per compute unit, all of which must be resident at once,
 * so other work that holds compute units for long while it runs can trip the wait limit.  Calls
 * that share a workspace or the state arrays must not overlap in time.
 */
typedef enum { REMOE_DECODE_CHAINED = 0, REMOE_DECODE_PIPELINED = 1 } remoe_decode_order;

size_t remoe_decode_workspace_bytes(const remoe_layer_desc *desc);
remoe_status moe_decode(const remoe_layer_desc *desc, int32_t n_layers,
                        const void *const *layer_weights,
                        const void *x, int64_t steps_total, int64_t step0, int64_t n_steps,
                        void *y, int32_t *out_idx, float *out_w,
                        int32_t n_caps, const int32_t *capacities, uint64_t expert_bytes,
                        uint32_t *lru_state, uint8_t *out_overlap, uint8_t *out_miss,
                        uint64_t *sum_overlap, uint64_t *total_miss, uint64_t *bytes_fetched,
                        void *workspace, size_t workspace_bytes, uint64_t spin_limit_us,
                        int32_t layer_order, void *stream);

/*
 * moe_decode_static -- moe_decode for callers that cannot allocate device memory or hand over a
 * workspace: code that runs under HIP graph capture, serving loops that must not touch the
 * allocator, harnesses that forbid hipMalloc.  It takes no workspace.  The kernels' scratch (abort
 * word, barrier flags, exchange rings) lives in a static device array inside the library of
 * remoe_decode_static_bytes() = 2,625,792 bytes, which every GPU the library runs on holds until
 * the process ends; that size covers every layer shape moe_decode accepts (a shape that needed
 * more is refused with REMOE_E_WORKSPACE).  The call allocates and frees nothing, on the host side
 * of the runtime or the device.
 *
 * Arguments, outputs, limits and error behaviour are those of moe_decode, with one addition:
 *   out_abort   DEVICE pointer to one uint32 owned by the caller; after the call it holds the abort
 *               word (non-zero: a wait inside the kernel exceeded `spin_limit_us`, the outputs of
 *               this call are invalid).
 *
 * All calls on one GPU share that GPU's array, whatever their stream: calls that overlap in time on
 * one GPU race on it and must be serialised by the caller.  The array keeps the previous call's
 * contents; the flags and exchange words are cleared by a kernel at the start of every call.
 */
size_t remoe_decode_static_bytes(void);
remoe_status moe_decode_static(const remoe_layer_desc *desc, int32_t n_layers,
                               const void *const *layer_weights,
                               const void *x, int64_t steps_total, int64_t step0, int64_t n_steps,
                               void *y, int32_t *out_idx, float *out_w,
                               int32_t n_caps, const int32_t *capacities, uint64_t expert_bytes,
                               uint32_t *lru_state, uint8_t *out_overlap, uint8_t *out_miss,
                               uint64_t *sum_overlap, uint64_t *total_miss, uint64_t *bytes_fetched,
                               uint32_t *out_abort, uint64_t spin_limit_us,
                               int32_t layer_order, void *stream);

/*
 * cache_simulate -- the paper's expert-cache simulator for the replacement policies it reports
 * besides LRU (App. E.2 "Cache state": LRU / LFU / FIFO; App. F.1: Belady's MIN under the same
 * per-request resets).  One cold cache of `capacity` experts per trace.  Per step, against the
 * resident set BEFORE the step (App. E.2, "Per-step hits and misses"):
 *
 *   out_miss[s, t]    = |U_t \ C_t|   unique misses           out_uniq[s, t] = |U_t|
 *   out_hit_tok[s, t] = number of routed slots (with multiplicity) whose expert is resident
 *   out_total_miss[s] = sum_t out_miss   (#uMiss)      out_total_uniq[s] = sum_t out_uniq
 *   out_bytes[s]      = out_total_miss[s] * expert_bytes       (uHR = 1 - total_miss / total_uniq)
 *
 * After the step every requested expert is held (App. A: the cache admits what the step fetched, and
 * what it used is resident when the next step starts); while more than `capacity` are held, one
 * expert is dropped: the one its policy ranks last among the held experts that this step did NOT
 * request, and only when no such expert is left (more distinct requests than `capacity`) the one
 * ranked last among the requested ones.  The rankings (the paper names the policies only; these are
 * the rules taken):
 *   REMOE_CACHE_LRU     least recently used; inside one step the higher id counts as later
 *   REMOE_CACHE_FIFO    earliest fetched (a hit does not renew); inside one step the higher id is later
 *   REMOE_CACHE_LFU     fewest requesting steps so far in the trace (kept across evictions), then
 *                       least recently used
 *   REMOE_CACHE_BELADY  next request farthest ahead (never again = farthest), then the higher id;
 *                       needs a workspace of remoe_cache_workspace_bytes() for the next-request table
 *
 *   idx [S, T, K] int32; n_experts <= 128, top_k <= 64, capacity >= 1, n_steps < 2^24.
 *   All pointers are device pointers; workspace may be NULL when no bytes are needed.
 */
typedef enum { REMOE_CACHE_LRU = 0, REMOE_CACHE_FIFO = 1, REMOE_CACHE_LFU = 2, REMOE_CACHE_BELADY = 3 } remoe_cache_policy;

size_t remoe_cache_workspace_bytes(int64_t n_seq, int64_t n_steps, int32_t top_k, int32_t policy);
remoe_status cache_simulate(const int32_t *idx, int64_t n_seq, int64_t n_steps, int32_t top_k,
                            int32_t n_experts, int32_t capacity, int32_t policy, uint64_t expert_bytes,
                            uint8_t *out_miss, uint8_t *out_uniq, uint8_t *out_hit_tok,
                            uint64_t *out_total_miss, uint64_t *out_total_uniq, uint64_t *out_bytes,
                            void *workspace, size_t workspace_bytes, void *stream);

/*
 * step_miss_summary -- per-step aggregates across all MoE layers and their percentiles (App. E.2,
 * "Per-step (edge) reporting"):
 *
 *   out_all[s, t] = sum over layers l of miss[l, s, t]                (#uMiss^(all)_{s,t})
 *   out_hist[v]   = number of steps (s, t) with out_all = v; sums >= hist_len share the last bin
 *   out_pct[0..2] = P50, P95, P99 of out_all over all steps: the smallest value whose cumulative
 *                   count reaches that percentage of the steps (-1 when there are no steps)
 *
 *   miss [L, S, T] uint8 (e.g. out_miss of lru_simulate / cache_simulate for every layer);
 *   out_all [S, T] uint16; out_hist [hist_len] uint64, 1 <= hist_len <= 4097; out_pct [3] int32.
 */
remoe_status step_miss_summary(const uint8_t *miss, int64_t n_layers, int64_t n_seq, int64_t n_steps,
                               uint16_t *out_all, uint64_t *out_hist, int64_t hist_len,
                               int32_t *out_pct, void *stream);

/*
 * routing_balance -- how evenly a trace spreads its routed slots over the experts (the routing
 * entropy, load variation and experts used that Sec. 5.2 tracks; the paper does not spell the
 * formulas out, these are the ones taken).  With load[e] = number of slots (t, j) that name expert
 * e and p_e = load[e] / (T K):
 *
 *   out_entropy[s] = -sum_e p_e ln p_e / ln N_r      (1 = even, 0 = a single expert; 0 if N_r = 1)
 *   out_cv[s]      = sqrt(mean_e (load[e] - m)^2) / m,  m = T K / N_r     (population form)
 *   out_used[s]    = number of experts with load > 0
 *
 *   idx [S, T, K] int32; out_load [S, N_r] uint32; out_used [S] int32; out_entropy, out_cv [S]
 *   double (computed in fp64).  n_experts <= 128.  Empty traces give 0, 0, 0.
 */
remoe_status routing_balance(const int32_t *idx, int64_t n_seq, int64_t n_steps, int32_t top_k,
                             int32_t n_experts, uint32_t *out_load, int32_t *out_used,
                             double *out_entropy, double *out_cv, void *stream);

/*
 * reroute_lru -- cache-aware rerouting at inference time (App. G, "Setup"): experts that are in the
 * per-layer LRU cache get a residency bonus beta on their pre-top-k router score; beta = 0 is the
 * unmodified router.  Routing and cache state depend on each other, so every trace is one
 * sequential pass from a cold cache.
 *
 *   score_t[e]  = probs[s, t, e] * factor   if e is resident before step t,  else probs[s, t, e]
 *                 (factor = exp(beta): the same order as adding beta to the resident experts' logits;
 *                 one fp32 multiply, so the selection is decided in fp32)
 *   out_idx[s, t, :]  the K experts of largest score, descending, ties to the lower id
 *   out_w[s, t, j]    probs[s, t, out_idx[s, t, j]] (the unmodified probability), divided by the
 *                     sum over the K chosen when renorm
 *   out_miss[s, t]    |E_t \ C_t| against the cache before the step; then E_t becomes the most
 *                     recent (ascending id inside the step) and the cache keeps `capacity` experts
 *   out_total_miss[s] sum_t out_miss[s, t]      (uHR = 1 - total_miss / (K T))
 *
 *   probs [S, T, N_r] fp32 (e.g. out_probs of moe_route); out_idx int32 [S, T, K]; out_w fp32 [S, T, K];
 *   out_miss uint8 [S, T]; out_total_miss uint64 [S].  n_experts <= 128, top_k <= min(n_experts, 64),
 *   capacity >= 1, factor > 0 and finite, n_steps < 2^24.
 */
remoe_status reroute_lru(const float *probs, int64_t n_seq, int64_t n_steps, int32_t n_experts, int32_t top_k,
                         int32_t capacity, float factor, int32_t renorm, int32_t *out_idx, float *out_w,
                         uint8_t *out_miss, uint64_t *out_total_miss, void *stream);

/*
 * remoe_loss_forward -- forward values of the router regularisers ReMoE trains with (Sec. 4.2-4.4),
 * per sequence, from the routing distributions of the trainable router (probs), of the frozen
 * snapshot router (probs_ref) and the routed sets (idx; the previous step's set is a constant of
 * the reuse mass):
 *
 *   out[s, 0] rho      = mean_{t>=2} m_t,  m_t = (1/K) sum_{k in E_{t-1}} P_t[k]          (Eq. 2, 7)
 *   out[s, 1] L_Reuse  = -log(rho + 1e-8)                                                 (Eq. 7)
 *   out[s, 2] L_Trust  = mean_t KL(P_t || P_t^ref)                                        (Eq. 5)
 *   out[s, 3] L_Smooth = mean_{t>=2} SymKL(P_t, P_{t-1})                                  (Eq. 9)
 *   out[s, 4] L_Lag    = mean_{t>=2} (1/|D|) sum_{d in D, t-d>=1} SymKL(P_t, P_{t-d})     (Eq. 10)
 *   out[s, 5] L_WS     = mean over the floor(T/W) windows of H(window mean of P)          (Eq. 12)
 *
 * The weighted sums L_Loc (Eq. 6) and L (Eq. 3) and the warm-up factor are left to the caller.
 * Conventions: 0 log 0 = 0; a sequence of one step has rho = 0 and no smoothness / lag term; no
 * full window gives L_WS = 0.  Computed in fp64 from the fp32 probabilities.
 *
 *   probs, probs_ref [S, T, N_r] fp32 (out_probs of moe_route with the two gate matrices);
 *   idx [S, T, K] int32; lags HOST array of n_lags (0..8) positive lags D; window W >= 1;
 *   out [S, 6] double; workspace remoe_loss_workspace_bytes(S) bytes, 8-byte aligned.
 *   n_experts <= 128, top_k <= 64, S <= 65535.
 */
size_t remoe_loss_workspace_bytes(int64_t n_seq);
remoe_status remoe_loss_forward(const float *probs, const float *probs_ref, const int32_t *idx,
                                int64_t n_seq, int64_t n_steps, int32_t n_experts, int32_t top_k,
                                const int32_t *lags, int32_t n_lags, int32_t window, double *out,
                                void *workspace, size_t workspace_bytes, void *stream);

/*
 * remoe_loss_backward -- gradient of the weighted sum of the regularisers above with respect to the
 * router logits (the backward pass of the gate-only fine-tuning step, Sec. 4.1 step 3; Eq. 3, 6):
 *
 *   L[s] = coef[0] L_Reuse + coef[1] L_Trust + coef[2] L_Smooth + coef[3] L_Lag + coef[4] L_WS,
 *   dlogits[s, t, k] = dL[s] / dz[s, t, k]   with P_t = softmax(z_t):
 *                      P_t[k] (g[k] - sum_j P_t[j] g[j]),  g = dL[s] / dP_t entry by entry.
 *
 * The previous routed set in the reuse mass and the snapshot router's distribution are constants
 * (stop-gradient, Eq. 2 and Eq. 4); both arguments of every SymKL carry gradient (Sec. 4.4 says so
 * for L_Smooth; taken for L_Lag as well).  Entries with P_t[k] = 0 get 0.  Computed in fp64 from
 * the fp32 probabilities, stored as fp32.  Sequences are independent: a mean over sequences is a
 * factor 1/S in coef.
 *
 *   probs, probs_ref, idx, lags, n_lags, window   as for remoe_loss_forward
 *   coef          HOST array of 5 doubles (warm-up factor and the lambdas of Eq. 3, 6 folded in)
 *   loss_values   DEVICE [S, 6] double: the output of remoe_loss_forward on the same inputs (rho is
 *                 read from it)
 *   dlogits       DEVICE [S, T, N_r] fp32, written
 *   workspace     remoe_loss_backward_workspace_bytes(S, T, N_r, window) bytes, 8-byte aligned
 *
 * remoe_gate_grad -- the gate gradient of a router without bias (Sec. 3.1: z_t = W_r x_t):
 *   dw[e, h] = sum_t dlogits[t, e] x[t, h]        (fp32 matrix cores, fp32 accumulation; the sum over
 *   tokens is split into chunks whose partial results are added in a fixed order: results repeat
 *   bit for bit)
 *   dlogits [T, N_r] fp32 (all sequences flattened); x [T, H] of x_dtype (REMOE_F32 / REMOE_BF16);
 *   dw [N_r, H] fp32, overwritten; workspace remoe_gate_grad_workspace_bytes(T, N_r, H) bytes,
 *   256-byte aligned.  n_experts <= 128, hidden % 64 == 0.
 */
size_t remoe_loss_backward_workspace_bytes(int64_t n_seq, int64_t n_steps, int32_t n_experts, int32_t window);
remoe_status remoe_loss_backward(const float *probs, const float *probs_ref, const int32_t *idx,
                                 int64_t n_seq, int64_t n_steps, int32_t n_experts, int32_t top_k,
                                 const int32_t *lags, int32_t n_lags, int32_t window, const double *coef,
                                 const double *loss_values, float *dlogits,
                                 void *workspace, size_t workspace_bytes, void *stream);
size_t remoe_gate_grad_workspace_bytes(int64_t n_tokens, int32_t n_experts, int32_t hidden);
remoe_status remoe_gate_grad(const float *dlogits, const void *x, int32_t x_dtype, int64_t n_tokens,
                             int32_t n_experts, int32_t hidden, float *dw,
                             void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* REMOE_H */
