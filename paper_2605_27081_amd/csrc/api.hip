// C-ABI entry points: argument validation, workspace layout and kernel sequencing.
#include <stdarg.h>
#include <string.h>

#include <mutex>
#include <utility>
#include <vector>

#include "common.h"

namespace remoe {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
}

remoe_status fail(remoe_status code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

remoe_status check_hip(hipError_t e, const char *what)
{
    if (e == hipSuccess) return REMOE_OK;
    return fail(REMOE_E_HIP, "%s: %s", what, hipGetErrorString(e));
}

// ---- optional per-kernel timing (benchmarks only) --------------------------------------------
// When enabled, every kernel group an entry point launches is bracketed by a pair of HIP events on
// the caller's stream; remoe_profile_read sums the elapsed times per kind.  Off by default: the
// entry points then record nothing.  The events come from a pool that remoe_profile_enable fills
// (PROF_POOL pairs, created once); the entry points themselves never create one, and a scope that
// finds the pool empty is simply not recorded.
namespace {

struct ProfRecord { int kind; hipEvent_t start, stop; };
std::mutex g_prof_mutex;
bool g_prof_on = false;
std::vector<ProfRecord> g_prof_used;
std::vector<std::pair<hipEvent_t, hipEvent_t>> g_prof_free;
constexpr size_t PROF_POOL = 4096;      // event pairs; enough for a dozen profiled passes over 48 layers

class ProfScope {
public:
    ProfScope(int kind, hipStream_t stream) : stream_(stream)
    {
        std::lock_guard<std::mutex> lock(g_prof_mutex);
        if (!g_prof_on) return;
        if (g_prof_free.empty()) return;      // pool used up: this scope goes unrecorded (nothing is created here)
        ProfRecord r{kind, g_prof_free.back().first, g_prof_free.back().second};
        g_prof_free.pop_back();
        if (hipEventRecord(r.start, stream_) != hipSuccess) return;
        rec_ = r;
        active_ = true;
    }
    ~ProfScope()
    {
        if (!active_) return;
        std::lock_guard<std::mutex> lock(g_prof_mutex);
        (void)hipEventRecord(rec_.stop, stream_);
        g_prof_used.push_back(rec_);
    }
private:
    hipStream_t stream_;
    ProfRecord rec_{};
    bool active_ = false;
};

}  // namespace

namespace {

constexpr int MAX_EXPERTS = 128;
constexpr int MAX_TOP_K = 8;
constexpr int64_t MAX_TOKENS = 1 << 22;   // keeps T*K and every slot index inside int32

remoe_status validate_route_desc(const remoe_layer_desc *d)
{
    if (!d) return fail(REMOE_E_INVALID_ARG, "desc is NULL");
    if (d->dtype != REMOE_F32 && d->dtype != REMOE_BF16)
        return fail(REMOE_E_INVALID_ARG, "dtype %d is neither REMOE_F32 nor REMOE_BF16", d->dtype);
    if (d->n_experts < 1 || d->n_experts > MAX_EXPERTS)
        return fail(REMOE_E_INVALID_ARG, "n_experts %d outside 1..%d", d->n_experts, MAX_EXPERTS);
    if (d->top_k < 1 || d->top_k > MAX_TOP_K || d->top_k > d->n_experts)
        return fail(REMOE_E_INVALID_ARG, "top_k %d outside 1..min(n_experts, %d)", d->top_k, MAX_TOP_K);
    if (d->hidden < 32 || d->hidden % 32 != 0)
        return fail(REMOE_E_INVALID_ARG, "hidden %d must be a positive multiple of 32", d->hidden);
    if (d->renorm != 0 && d->renorm != 1) return fail(REMOE_E_INVALID_ARG, "renorm must be 0 or 1");
    return REMOE_OK;
}

remoe_status validate_layer_desc(const remoe_layer_desc *d)
{
    remoe_status st = validate_route_desc(d);
    if (st != REMOE_OK) return st;
    if (d->inter < 1) return fail(REMOE_E_INVALID_ARG, "inter %d must be positive", d->inter);
    if (d->shared_inter < 0) return fail(REMOE_E_INVALID_ARG, "shared_inter %d is negative", d->shared_inter);
    if (d->shared_gate != 0 && d->shared_gate != 1)
        return fail(REMOE_E_INVALID_ARG, "shared_gate must be 0 or 1");
    if (d->shared_gate && d->shared_inter == 0)
        return fail(REMOE_E_INVALID_ARG, "shared_gate set without a shared expert");
    if (d->dtype == REMOE_BF16) {
        if (d->hidden % 128 != 0)
            return fail(REMOE_E_UNSUPPORTED, "bf16 layers need hidden %% 128 == 0 (got %d)", d->hidden);
        if (d->inter % 64 != 0 || d->shared_inter % 64 != 0)
            return fail(REMOE_E_UNSUPPORTED, "bf16 layers need inter and shared_inter %% 64 == 0 (got %d, %d)",
                        d->inter, d->shared_inter);
    }
    return REMOE_OK;
}

// Workspace carving, shared by remoe_workspace_bytes and moe_forward.
struct Workspace {
    size_t total = 0;
    PermuteBuffers pb{};
    void *hbuf = nullptr;     // [T*K, I]            SwiGLU activations of the routed experts
    void *hsbuf = nullptr;    // [T, I_s]            SwiGLU activations of the shared expert
    void *rows = nullptr;     // [T*K (+T), H]       weighted per-(token, expert) outputs, then shared rows
    int max_tiles = 0;
};

template <typename P> void carve(char *base, size_t &off, P *&ptr, size_t bytes)
{
    off = align_up(off, 256);
    ptr = base ? reinterpret_cast<P *>(base + off) : nullptr;
    off += bytes;
}

Workspace layout(const remoe_layer_desc *d, int64_t T, void *base_v)
{
    Workspace w;
    char *base = static_cast<char *>(base_v);
    const size_t es = d->dtype == REMOE_F32 ? 4 : 2;
    const int64_t pairs = T * d->top_k;
    const int64_t n_blk = ceil_div(T, permute_tokens_per_block());
    w.max_tiles = (int)(ceil_div(pairs, gemm_tile_m()) + d->n_experts);
    size_t off = 0;
    carve(base, off, w.pb.blk_hist, sizeof(int32_t) * 2 * n_blk * d->n_experts);
    carve(base, off, w.pb.offsets, sizeof(int32_t) * (d->n_experts + 1));
    carve(base, off, w.pb.tile_expert, sizeof(int32_t) * w.max_tiles);
    carve(base, off, w.pb.tile_row0, sizeof(int32_t) * w.max_tiles);
    carve(base, off, w.pb.tile_rows, sizeof(int32_t) * w.max_tiles);
    carve(base, off, w.pb.n_tiles, sizeof(int32_t));
    carve(base, off, w.pb.gemm_ctr, sizeof(uint32_t) * GEMM_CTR_SETS * 8);
    carve(base, off, w.pb.pair_slot, sizeof(int32_t) * pairs);
    carve(base, off, w.pb.slot_token, sizeof(int32_t) * pairs);
    carve(base, off, w.pb.slot_w, sizeof(float) * pairs);
    carve(base, off, w.hbuf, es * pairs * d->inter);
    carve(base, off, w.hsbuf, es * T * d->shared_inter);
    carve(base, off, w.rows, es * (pairs + (d->shared_inter ? T : 0)) * d->hidden);
    w.total = align_up(off, 256);
    return w;
}

// ---- scratch of moe_decode_static -------------------------------------------------------------
// Callers that cannot allocate (code under graph capture, serving loops) get the decode kernels'
// scratch (abort word, barrier flags, rings of exchange words) from this array instead of a
// workspace argument.  Its size covers every layer shape moe_decode supports: n_experts <= 128,
// hidden <= 4096, top_k * inter <= 6144 give 4352 bytes of flags + 8 groups x 4 ring slots x
// (2048 + 8192) eight-byte words.  Every GPU the library runs on holds its own copy until the
// process ends.  In host code the array's name is only a handle for hipGetSymbolAddress: the
// device address it yields (one per device) is what the kernels and the host-side layout use.
constexpr size_t DECODE_STATIC_BYTES = 4352 + (size_t)8 * 4 * (2048 + 8192) * 8;
static __device__ __align__(256) unsigned char g_decode_scratch[DECODE_STATIC_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_decode_scratch_ptr[MAX_DEVICES] = {};

// device address of g_decode_scratch on the current device (looked up once per device)
remoe_status decode_static_scratch(void **out)
{
    int dev = -1;
    REMOE_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(REMOE_E_UNSUPPORTED, "device ordinal %d outside 0..%d", dev, MAX_DEVICES - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_decode_scratch_ptr[dev]) {
        void *ptr = nullptr;
        REMOE_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_decode_scratch)));
        if (!ptr || ((uintptr_t)ptr & 255)) return fail(REMOE_E_HIP, "static decode scratch has no usable device address");
        g_decode_scratch_ptr[dev] = ptr;
    }
    *out = g_decode_scratch_ptr[dev];
    return REMOE_OK;
}

__global__ void copy_abort_word_kernel(const uint32_t *src, uint32_t *dst) { *dst = src ? *src : 0u; }

}  // namespace
}  // namespace remoe

using namespace remoe;

extern "C" {
#pragma GCC visibility push(default)

int32_t remoe_version(void) { return 100; }

const char *remoe_last_error(void) { return g_err; }

remoe_status remoe_profile_enable(int32_t on)
{
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (on) {
        while (g_prof_free.size() + g_prof_used.size() < PROF_POOL) {
            hipEvent_t a = nullptr, b = nullptr;
            if (hipEventCreate(&a) != hipSuccess) return fail(REMOE_E_HIP, "hipEventCreate failed while filling the timing pool");
            if (hipEventCreate(&b) != hipSuccess) {
                (void)hipEventDestroy(a);
                return fail(REMOE_E_HIP, "hipEventCreate failed while filling the timing pool");
            }
            g_prof_free.emplace_back(a, b);
        }
    }
    g_prof_on = on != 0;
    return REMOE_OK;
}

remoe_status remoe_profile_read(int32_t kind, double *total_ms, int64_t *launches, int32_t reset)
{
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (kind < 0 || kind >= REMOE_PROF_KINDS) return fail(REMOE_E_INVALID_ARG, "profile kind %d out of range", kind);
    double sum = 0.0;
    int64_t n = 0;
    for (const ProfRecord &r : g_prof_used) {
        if (r.kind != kind) continue;
        float ms = 0.f;
        hipError_t e = hipEventElapsedTime(&ms, r.start, r.stop);
        if (e != hipSuccess) return check_hip(e, "hipEventElapsedTime (synchronise the stream before reading)");
        sum += ms;
        ++n;
    }
    if (total_ms) *total_ms = sum;
    if (launches) *launches = n;
    if (reset) {
        std::vector<ProfRecord> keep;
        for (const ProfRecord &r : g_prof_used) {
            if (r.kind == kind) g_prof_free.emplace_back(r.start, r.stop);
            else keep.push_back(r);
        }
        g_prof_used.swap(keep);
    }
    return REMOE_OK;
}

remoe_status remoe_copy_probe(void *dst, const void *src, size_t bytes, void *stream)
{
    if (bytes == 0) return REMOE_OK;
    if (!dst || !src) return fail(REMOE_E_INVALID_ARG, "dst and src must not be NULL");
    if ((bytes & 15) || (((uintptr_t)dst | (uintptr_t)src) & 15))
        return fail(REMOE_E_INVALID_ARG, "copy probe needs 16-byte aligned pointers and a multiple of 16 bytes");
    const uintptr_t d = (uintptr_t)dst, s = (uintptr_t)src;
    if (d < s + bytes && s < d + bytes) return fail(REMOE_E_INVALID_ARG, "copy probe ranges overlap");
    return launch_copy_probe(dst, src, bytes, static_cast<hipStream_t>(stream));
}

size_t remoe_workspace_bytes(const remoe_layer_desc *desc, int64_t n_tokens)
{
    if (validate_layer_desc(desc) != REMOE_OK) return 0;
    if (n_tokens < 0 || n_tokens > MAX_TOKENS) {
        set_error("n_tokens %lld outside 0..%lld", (long long)n_tokens, (long long)MAX_TOKENS);
        return 0;
    }
    return layout(desc, n_tokens, nullptr).total;
}

remoe_status moe_route(const remoe_layer_desc *desc, const void *x, int64_t n_tokens,
                       const float *w_router, int32_t *out_idx, float *out_w, float *out_margin,
                       float *out_probs, void *stream)
{
    remoe_status st = validate_route_desc(desc);
    if (st != REMOE_OK) return st;
    if (n_tokens < 0 || n_tokens > MAX_TOKENS)
        return fail(REMOE_E_INVALID_ARG, "n_tokens %lld outside 0..%lld", (long long)n_tokens, (long long)MAX_TOKENS);
    if (n_tokens == 0) return REMOE_OK;
    if (!x || !w_router || !out_idx || !out_w)
        return fail(REMOE_E_INVALID_ARG, "x, w_router, out_idx and out_w must not be NULL");
    if (((uintptr_t)x | (uintptr_t)w_router) & 15)
        return fail(REMOE_E_INVALID_ARG, "x and w_router must be 16-byte aligned");
    ProfScope prof(REMOE_PROF_ROUTE, static_cast<hipStream_t>(stream));
    return launch_route(x, desc->dtype, n_tokens, desc->hidden, w_router, desc->n_experts, desc->top_k,
                        desc->renorm, out_idx, out_w, out_margin, out_probs, static_cast<hipStream_t>(stream));
}

remoe_status moe_forward(const remoe_layer_desc *desc, const void *x, int64_t n_tokens,
                         const float *w_router, const void *w_gate, const void *w_up,
                         const void *w_down, const void *ws_gate, const void *ws_up,
                         const void *ws_down, const float *ws_scale, void *y, int32_t *out_idx,
                         float *out_w, void *workspace, size_t workspace_bytes, void *stream_v)
{
    remoe_status st = validate_layer_desc(desc);
    if (st != REMOE_OK) return st;
    const int64_t T = n_tokens;
    if (T < 0 || T > MAX_TOKENS)
        return fail(REMOE_E_INVALID_ARG, "n_tokens %lld outside 0..%lld", (long long)T, (long long)MAX_TOKENS);
    if (T == 0) return REMOE_OK;
    if (!x || !w_router || !w_gate || !w_up || !w_down || !y || !out_idx || !out_w)
        return fail(REMOE_E_INVALID_ARG, "a required pointer is NULL");
    if (desc->shared_inter > 0 && (!ws_gate || !ws_up || !ws_down))
        return fail(REMOE_E_INVALID_ARG, "shared_inter > 0 but a shared-expert matrix is NULL");
    if (desc->shared_gate && !ws_scale)
        return fail(REMOE_E_INVALID_ARG, "shared_gate set but ws_scale is NULL");
    const uintptr_t all = (uintptr_t)x | (uintptr_t)w_router | (uintptr_t)w_gate | (uintptr_t)w_up |
                          (uintptr_t)w_down | (uintptr_t)ws_gate | (uintptr_t)ws_up |
                          (uintptr_t)ws_down | (uintptr_t)ws_scale | (uintptr_t)y;
    if (all & 15) return fail(REMOE_E_INVALID_ARG, "tensors must be 16-byte aligned");
    if (!workspace || ((uintptr_t)workspace & 255))
        return fail(REMOE_E_WORKSPACE, "workspace is NULL or not 256-byte aligned");
    const Workspace ws = layout(desc, T, workspace);
    if (workspace_bytes < ws.total)
        return fail(REMOE_E_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, ws.total);

    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    const int H = desc->hidden, I = desc->inter, Is = desc->shared_inter, K = desc->top_k, N = desc->n_experts;
    const bool f32 = desc->dtype == REMOE_F32;
    auto gemm = [&](int mode, const GroupedGemmArgs &g) {
        return f32 ? launch_grouped_gemm_f32(mode, g, stream) : launch_grouped_gemm_bf16(mode, g, stream);
    };

    // 1. router: logits, top-k, softmax weights
    {
        ProfScope prof(REMOE_PROF_ROUTE, stream);
        st = launch_route(x, desc->dtype, T, H, w_router, N, K, desc->renorm, out_idx, out_w, nullptr, nullptr, stream);
    }
    if (st != REMOE_OK) return st;
    // 2. sort (token, j) pairs by expert; build the GEMM tile list
    {
        ProfScope prof(REMOE_PROF_PERMUTE, stream);
        st = launch_permute(out_idx, out_w, T, K, N, gemm_tile_m(), ws.max_tiles, ws.pb, stream);
    }
    if (st != REMOE_OK) return st;
    // 3. routed experts: gate/up + SwiGLU, then the down projection (the fp32 kernel also applies the gate weight)
    GroupedGemmArgs g{};
    g.a = x; g.lda = H; g.a_rows = T; g.row_gather = ws.pb.slot_token;
    g.b0 = w_gate; g.b1 = w_up; g.k_dim = H; g.n_out = I;
    g.tile_expert = ws.pb.tile_expert; g.tile_row0 = ws.pb.tile_row0; g.tile_rows = ws.pb.tile_rows;
    g.n_tiles = ws.pb.n_tiles; g.max_tiles = ws.max_tiles;
    g.c = ws.hbuf; g.ldc = I; g.c_row_offset = 0;
    g.tile_ctr = ws.pb.gemm_ctr;
    {
        ProfScope prof(REMOE_PROF_GATE_UP, stream);
        st = gemm(0, g);
    }
    if (st != REMOE_OK) return st;
    g.a = ws.hbuf; g.lda = I; g.a_rows = T * K; g.row_gather = nullptr;
    g.b0 = w_down; g.b1 = nullptr; g.k_dim = I; g.n_out = H;
    g.row_scale = f32 ? ws.pb.slot_w : nullptr;   // bf16: the combine step applies the gate weights
    g.c = ws.rows; g.ldc = H;
    g.tile_ctr = ws.pb.gemm_ctr + 8;
    {
        ProfScope prof(REMOE_PROF_DOWN, stream);
        st = gemm(1, g);
    }
    if (st != REMOE_OK) return st;
    // 4. shared expert (dense, one group): rows T*K .. T*K+T-1 of the row buffer
    if (Is > 0) {
        GroupedGemmArgs s{};
        s.a = x; s.lda = H; s.a_rows = T; s.b0 = ws_gate; s.b1 = ws_up; s.k_dim = H; s.n_out = Is;
        s.dense_rows = T; s.max_tiles = (int)ceil_div(T, gemm_tile_m());
        s.c = ws.hsbuf; s.ldc = Is;
        s.tile_ctr = ws.pb.gemm_ctr + 16;
        {
            ProfScope prof(REMOE_PROF_SHARED_GATE_UP, stream);
            st = gemm(0, s);
        }
        if (st != REMOE_OK) return st;
        s.a = ws.hsbuf; s.lda = Is; s.a_rows = T; s.b0 = ws_down; s.b1 = nullptr; s.k_dim = Is; s.n_out = H;
        s.c = ws.rows; s.ldc = H; s.c_row_offset = T * K;
        s.tile_ctr = ws.pb.gemm_ctr + 24;
        {
            ProfScope prof(REMOE_PROF_SHARED_DOWN, stream);
            st = gemm(1, s);
        }
        if (st != REMOE_OK) return st;
    }
    // 5. combine the K (+1) rows of every token
    ProfScope prof(REMOE_PROF_COMBINE, stream);
    return launch_combine(desc->dtype, ws.rows, ws.pb.pair_slot, f32 ? nullptr : out_w, T, K, H, T * K, Is > 0, x,
                          desc->shared_gate ? ws_scale : nullptr, y, stream);
}

static remoe_status validate_trace(const int32_t *idx, int64_t n_seq, int64_t n_steps, int32_t top_k,
                                   int32_t n_experts)
{
    if (n_seq < 0 || n_steps < 0) return fail(REMOE_E_INVALID_ARG, "negative trace dimensions");
    if (n_seq > 0x7FFFFFFF) return fail(REMOE_E_INVALID_ARG, "n_seq %lld too large", (long long)n_seq);
    if (n_experts < 1 || n_experts > MAX_EXPERTS)
        return fail(REMOE_E_INVALID_ARG, "n_experts %d outside 1..%d", n_experts, MAX_EXPERTS);
    if (top_k < 1 || top_k > 64) return fail(REMOE_E_INVALID_ARG, "top_k %d outside 1..64", top_k);
    if (n_seq > 0 && n_steps > 0 && !idx) return fail(REMOE_E_INVALID_ARG, "idx is NULL");
    return REMOE_OK;
}

remoe_status trace_reuse(const int32_t *idx, int64_t n_seq, int64_t n_steps, int32_t top_k,
                         int32_t n_experts, uint8_t *out_overlap, uint64_t *out_sum, void *stream)
{
    remoe_status st = validate_trace(idx, n_seq, n_steps, top_k, n_experts);
    if (st != REMOE_OK) return st;
    if (n_seq == 0) return REMOE_OK;
    if (!out_sum || (n_steps > 0 && !out_overlap))
        return fail(REMOE_E_INVALID_ARG, "out_overlap and out_sum must not be NULL");
    ProfScope prof(REMOE_PROF_TRACE_REUSE, static_cast<hipStream_t>(stream));
    return launch_trace_reuse(idx, n_seq, n_steps, top_k, n_experts, out_overlap, out_sum,
                              static_cast<hipStream_t>(stream));
}

remoe_status lru_simulate(const int32_t *idx, int64_t n_seq, int64_t n_steps, int32_t top_k,
                          int32_t n_experts, int32_t capacity, uint64_t expert_bytes, int64_t step0,
                          uint32_t *state, uint8_t *out_miss, uint64_t *out_total_miss,
                          uint64_t *out_bytes, void *stream)
{
    if (capacity < 1) return fail(REMOE_E_INVALID_ARG, "capacity %d must be at least 1", capacity);
    if (step0 < 0 || n_steps < 0 || step0 + n_steps >= (1 << 24))
        return fail(REMOE_E_INVALID_ARG, "step0 + n_steps = %lld must stay in 0..2^24-1", (long long)(step0 + n_steps));
    remoe_status st = validate_trace(idx, n_seq, n_steps, top_k, n_experts);
    if (st != REMOE_OK) return st;
    if (n_seq == 0) return REMOE_OK;
    if (!out_total_miss || !out_bytes || (n_steps > 0 && !out_miss))
        return fail(REMOE_E_INVALID_ARG, "out_miss, out_total_miss and out_bytes must not be NULL");
    ProfScope prof(REMOE_PROF_LRU, static_cast<hipStream_t>(stream));
    return launch_lru(idx, n_seq, n_steps, top_k, n_experts, capacity, expert_bytes, step0, state, out_miss,
                      out_total_miss, out_bytes, static_cast<hipStream_t>(stream));
}

size_t remoe_decode_workspace_bytes(const remoe_layer_desc *desc)
{
    if (validate_layer_desc(desc) != REMOE_OK) return 0;
    return decode_workspace_bytes(desc->hidden, desc->n_experts, desc->inter, desc->top_k);
}

// moe_decode and moe_decode_static share everything but where the scratch memory comes from.
static remoe_status decode_impl(const remoe_layer_desc *desc, int32_t n_layers, const void *const *layer_weights,
                                const void *x, int64_t steps_total, int64_t step0, int64_t n_steps, void *y,
                                int32_t *out_idx, float *out_w, int32_t n_caps, const int32_t *capacities,
                                uint64_t expert_bytes, uint32_t *lru_state, uint8_t *out_overlap, uint8_t *out_miss,
                                uint64_t *sum_overlap, uint64_t *total_miss, uint64_t *bytes_fetched, void *workspace,
                                size_t workspace_bytes, uint64_t spin_limit_us, int32_t layer_order, void *stream)
{
    remoe_status st = validate_layer_desc(desc);
    if (st != REMOE_OK) return st;
    if (desc->dtype != REMOE_BF16 || desc->shared_inter != 0)
        return fail(REMOE_E_UNSUPPORTED, "moe_decode handles bf16 layers without a shared expert");
    if (n_layers < 1) return fail(REMOE_E_INVALID_ARG, "n_layers %d must be positive", n_layers);
    if (layer_order != REMOE_DECODE_CHAINED && layer_order != REMOE_DECODE_PIPELINED)
        return fail(REMOE_E_INVALID_ARG, "layer_order %d is neither REMOE_DECODE_CHAINED nor REMOE_DECODE_PIPELINED", layer_order);
    if (steps_total < 0 || step0 < 0 || n_steps < 0 || step0 + n_steps > steps_total || steps_total >= (1 << 24))
        return fail(REMOE_E_INVALID_ARG, "step range [%lld, %lld) outside 0..steps_total = %lld (< 2^24)",
                    (long long)step0, (long long)(step0 + n_steps), (long long)steps_total);
    if (n_caps < 0 || n_caps > 4) return fail(REMOE_E_INVALID_ARG, "n_caps %d outside 0..4", n_caps);
    if (n_caps > 0 && !capacities) return fail(REMOE_E_INVALID_ARG, "capacities is NULL");
    for (int c = 0; c < n_caps; ++c)
        if (capacities[c] < 1) return fail(REMOE_E_INVALID_ARG, "capacity %d must be at least 1", capacities[c]);
    if (n_steps == 0) return REMOE_OK;
    if (!layer_weights || !x || !y || !out_idx || !out_w || !lru_state || !out_overlap || !sum_overlap)
        return fail(REMOE_E_INVALID_ARG, "a required pointer is NULL");
    if (n_caps > 0 && (!out_miss || !total_miss || !bytes_fetched))
        return fail(REMOE_E_INVALID_ARG, "miss outputs are NULL");
    if (((uintptr_t)x | (uintptr_t)y) & 15) return fail(REMOE_E_INVALID_ARG, "x and y must be 16-byte aligned");
    if (!workspace || ((uintptr_t)workspace & 255))
        return fail(REMOE_E_WORKSPACE, "workspace is NULL or not 256-byte aligned");
    const size_t need = decode_workspace_bytes(desc->hidden, desc->n_experts, desc->inter, desc->top_k);
    if (workspace_bytes < need) return fail(REMOE_E_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);

    DecodeLaunch d{};
    d.layers = layer_weights;
    d.x = x;
    d.steps_total = steps_total; d.step0 = step0; d.n_steps = n_steps;
    d.n_layers = n_layers; d.H = desc->hidden; d.N = desc->n_experts; d.I = desc->inter; d.K = desc->top_k;
    d.renorm = desc->renorm;
    d.y = y; d.out_idx = out_idx; d.out_w = out_w;
    d.n_caps = n_caps;
    for (int c = 0; c < n_caps; ++c) d.caps[c] = capacities[c];
    d.expert_bytes = expert_bytes;
    d.lru_state = lru_state; d.out_overlap = out_overlap; d.out_miss = out_miss;
    d.sum_overlap = sum_overlap; d.total_miss = total_miss; d.bytes_fetched = bytes_fetched;
    d.workspace = workspace;
    d.spin_limit_ticks = (spin_limit_us ? spin_limit_us : 2000000ull) * 100ull;   // 100 MHz wall clock
    ProfScope prof(REMOE_PROF_DECODE, static_cast<hipStream_t>(stream));
    return layer_order == REMOE_DECODE_PIPELINED ? launch_decode_pipelined(d, static_cast<hipStream_t>(stream))
                                                 : launch_decode(d, static_cast<hipStream_t>(stream));
}

remoe_status moe_decode(const remoe_layer_desc *desc, int32_t n_layers, const void *const *layer_weights,
                        const void *x, int64_t steps_total, int64_t step0, int64_t n_steps, void *y,
                        int32_t *out_idx, float *out_w, int32_t n_caps, const int32_t *capacities,
                        uint64_t expert_bytes, uint32_t *lru_state, uint8_t *out_overlap, uint8_t *out_miss,
                        uint64_t *sum_overlap, uint64_t *total_miss, uint64_t *bytes_fetched, void *workspace,
                        size_t workspace_bytes, uint64_t spin_limit_us, int32_t layer_order, void *stream)
{
    return decode_impl(desc, n_layers, layer_weights, x, steps_total, step0, n_steps, y, out_idx, out_w, n_caps,
                       capacities, expert_bytes, lru_state, out_overlap, out_miss, sum_overlap, total_miss,
                       bytes_fetched, workspace, workspace_bytes, spin_limit_us, layer_order, stream);
}

size_t remoe_decode_static_bytes(void) { return DECODE_STATIC_BYTES; }

remoe_status moe_decode_static(const remoe_layer_desc *desc, int32_t n_layers, const void *const *layer_weights,
                               const void *x, int64_t steps_total, int64_t step0, int64_t n_steps, void *y,
                               int32_t *out_idx, float *out_w, int32_t n_caps, const int32_t *capacities,
                               uint64_t expert_bytes, uint32_t *lru_state, uint8_t *out_overlap, uint8_t *out_miss,
                               uint64_t *sum_overlap, uint64_t *total_miss, uint64_t *bytes_fetched,
                               uint32_t *out_abort, uint64_t spin_limit_us, int32_t layer_order, void *stream)
{
    remoe_status st = validate_layer_desc(desc);
    if (st != REMOE_OK) return st;
    if (!out_abort) return fail(REMOE_E_INVALID_ARG, "out_abort is NULL");
    const size_t need = decode_workspace_bytes(desc->hidden, desc->n_experts, desc->inter, desc->top_k);
    if (need > DECODE_STATIC_BYTES)
        return fail(REMOE_E_WORKSPACE, "moe_decode_static: this layer shape needs %zu bytes of scratch, the static "
                    "array holds %zu; use moe_decode with a workspace", need, (size_t)DECODE_STATIC_BYTES);
    void *scratch = nullptr;
    st = decode_static_scratch(&scratch);
    if (st != REMOE_OK) return st;
    st = decode_impl(desc, n_layers, layer_weights, x, steps_total, step0, n_steps, y, out_idx, out_w, n_caps,
                     capacities, expert_bytes, lru_state, out_overlap, out_miss, sum_overlap, total_miss,
                     bytes_fetched, scratch, DECODE_STATIC_BYTES, spin_limit_us, layer_order, stream);
    if (st != REMOE_OK) return st;
    // hand the abort word (byte 128 of the scratch) to the caller; a call that ran no step reports 0
    hipLaunchKernelGGL(copy_abort_word_kernel, dim3(1), dim3(1), 0, static_cast<hipStream_t>(stream),
                       n_steps > 0 ? reinterpret_cast<const uint32_t *>(static_cast<const char *>(scratch) + 128) : nullptr,
                       out_abort);
    return check_hip(hipGetLastError(), "moe_decode_static abort-word copy");
}

size_t remoe_cache_workspace_bytes(int64_t n_seq, int64_t n_steps, int32_t top_k, int32_t policy)
{
    if (n_seq < 0 || n_steps < 0 || top_k < 1) return 0;
    return cache_workspace_bytes(n_seq, n_steps, top_k, policy);
}

remoe_status cache_simulate(const int32_t *idx, int64_t n_seq, int64_t n_steps, int32_t top_k, int32_t n_experts,
                            int32_t capacity, int32_t policy, uint64_t expert_bytes, uint8_t *out_miss,
                            uint8_t *out_uniq, uint8_t *out_hit_tok, uint64_t *out_total_miss,
                            uint64_t *out_total_uniq, uint64_t *out_bytes, void *workspace, size_t workspace_bytes,
                            void *stream)
{
    if (capacity < 1) return fail(REMOE_E_INVALID_ARG, "capacity %d must be at least 1", capacity);
    if (policy < REMOE_CACHE_LRU || policy > REMOE_CACHE_BELADY)
        return fail(REMOE_E_INVALID_ARG, "unknown cache policy %d", policy);
    if (n_steps >= (1 << 24)) return fail(REMOE_E_INVALID_ARG, "n_steps %lld must stay below 2^24", (long long)n_steps);
    remoe_status st = validate_trace(idx, n_seq, n_steps, top_k, n_experts);
    if (st != REMOE_OK) return st;
    if (n_seq == 0) return REMOE_OK;
    if (!out_total_miss || !out_total_uniq || !out_bytes || (n_steps > 0 && (!out_miss || !out_uniq || !out_hit_tok)))
        return fail(REMOE_E_INVALID_ARG, "an output pointer is NULL");
    const size_t need = cache_workspace_bytes(n_seq, n_steps, top_k, policy);
    if (need > 0 && (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 15)))
        return fail(REMOE_E_WORKSPACE, "cache_simulate needs a 16-byte aligned workspace of %zu bytes for this policy", need);
    ProfScope prof(REMOE_PROF_CACHE, static_cast<hipStream_t>(stream));
    return launch_cache_policy(idx, n_seq, n_steps, top_k, n_experts, capacity, policy, expert_bytes, out_miss, out_uniq,
                               out_hit_tok, out_total_miss, out_total_uniq, out_bytes, workspace,
                               static_cast<hipStream_t>(stream));
}

remoe_status step_miss_summary(const uint8_t *miss, int64_t n_layers, int64_t n_seq, int64_t n_steps,
                               uint16_t *out_all, uint64_t *out_hist, int64_t hist_len, int32_t *out_pct, void *stream)
{
    if (n_layers < 0 || n_seq < 0 || n_steps < 0) return fail(REMOE_E_INVALID_ARG, "negative dimensions");
    if (n_layers > 257) return fail(REMOE_E_INVALID_ARG, "n_layers %lld: sums of uint8 over more than 257 layers do not fit uint16", (long long)n_layers);
    if (hist_len < 1 || hist_len > step_summary_max_hist())
        return fail(REMOE_E_INVALID_ARG, "hist_len %lld outside 1..%d", (long long)hist_len, step_summary_max_hist());
    if (!out_hist || !out_pct) return fail(REMOE_E_INVALID_ARG, "out_hist and out_pct must not be NULL");
    if (n_seq * n_steps > 0 && ((n_layers > 0 && !miss) || !out_all))
        return fail(REMOE_E_INVALID_ARG, "miss and out_all must not be NULL");
    return launch_step_summary(miss, n_layers, n_seq, n_steps, out_all, out_hist, (int)hist_len, out_pct,
                               static_cast<hipStream_t>(stream));
}

remoe_status routing_balance(const int32_t *idx, int64_t n_seq, int64_t n_steps, int32_t top_k, int32_t n_experts,
                             uint32_t *out_load, int32_t *out_used, double *out_entropy, double *out_cv, void *stream)
{
    remoe_status st = validate_trace(idx, n_seq, n_steps, top_k, n_experts);
    if (st != REMOE_OK) return st;
    if (n_seq == 0) return REMOE_OK;
    if (!out_load || !out_used || !out_entropy || !out_cv) return fail(REMOE_E_INVALID_ARG, "an output pointer is NULL");
    return launch_balance(idx, n_seq, n_steps, top_k, n_experts, out_load, out_used, out_entropy, out_cv,
                          static_cast<hipStream_t>(stream));
}

remoe_status reroute_lru(const float *probs, int64_t n_seq, int64_t n_steps, int32_t n_experts, int32_t top_k,
                         int32_t capacity, float factor, int32_t renorm, int32_t *out_idx, float *out_w,
                         uint8_t *out_miss, uint64_t *out_total_miss, void *stream)
{
    if (n_seq < 0 || n_steps < 0 || n_seq > 0x7FFFFFFF) return fail(REMOE_E_INVALID_ARG, "bad trace dimensions");
    if (n_steps >= (1 << 24)) return fail(REMOE_E_INVALID_ARG, "n_steps %lld must stay below 2^24", (long long)n_steps);
    if (n_experts < 1 || n_experts > MAX_EXPERTS) return fail(REMOE_E_INVALID_ARG, "n_experts %d outside 1..%d", n_experts, MAX_EXPERTS);
    if (top_k < 1 || top_k > n_experts || top_k > 64) return fail(REMOE_E_INVALID_ARG, "top_k %d outside 1..min(n_experts, 64)", top_k);
    if (capacity < 1) return fail(REMOE_E_INVALID_ARG, "capacity %d must be at least 1", capacity);
    if (!(factor > 0.0f) || factor > 3.0e38f) return fail(REMOE_E_INVALID_ARG, "factor must be positive and finite");
    if (n_seq == 0) return REMOE_OK;
    if (!out_total_miss || (n_steps > 0 && (!probs || !out_idx || !out_w || !out_miss)))
        return fail(REMOE_E_INVALID_ARG, "a required pointer is NULL");
    ProfScope prof(REMOE_PROF_CACHE, static_cast<hipStream_t>(stream));
    return launch_reroute(probs, n_seq, n_steps, n_experts, top_k, capacity, factor, renorm, out_idx, out_w, out_miss,
                          out_total_miss, static_cast<hipStream_t>(stream));
}

size_t remoe_loss_workspace_bytes(int64_t n_seq) { return n_seq < 0 ? 0 : loss_workspace_bytes(n_seq); }

remoe_status remoe_loss_forward(const float *probs, const float *probs_ref, const int32_t *idx, int64_t n_seq,
                                int64_t n_steps, int32_t n_experts, int32_t top_k, const int32_t *lags, int32_t n_lags,
                                int32_t window, double *out, void *workspace, size_t workspace_bytes, void *stream)
{
    remoe_status st = validate_trace(idx, n_seq, n_steps, top_k, n_experts);
    if (st != REMOE_OK) return st;
    if (n_lags < 0 || n_lags > 8 || (n_lags > 0 && !lags)) return fail(REMOE_E_INVALID_ARG, "n_lags %d outside 0..8 or lags is NULL", n_lags);
    for (int i = 0; i < n_lags; ++i)
        if (lags[i] < 1) return fail(REMOE_E_INVALID_ARG, "lag %d must be positive", lags[i]);
    if (window < 1) return fail(REMOE_E_INVALID_ARG, "window %d must be positive", window);
    if (n_seq == 0) return REMOE_OK;
    if (!out || (n_steps > 0 && (!probs || !probs_ref))) return fail(REMOE_E_INVALID_ARG, "a required pointer is NULL");
    const size_t need = loss_workspace_bytes(n_seq);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 7))
        return fail(REMOE_E_WORKSPACE, "remoe_loss_forward needs an 8-byte aligned workspace of %zu bytes", need);
    return launch_loss_forward(probs, probs_ref, idx, n_seq, n_steps, n_experts, top_k, lags, n_lags, window, out, workspace,
                               static_cast<hipStream_t>(stream));
}

size_t remoe_loss_backward_workspace_bytes(int64_t n_seq, int64_t n_steps, int32_t n_experts, int32_t window)
{
    if (n_seq < 0 || n_steps < 0 || n_experts < 1 || window < 1) return 0;
    return loss_backward_workspace_bytes(n_seq, n_steps, n_experts, window);
}

remoe_status remoe_loss_backward(const float *probs, const float *probs_ref, const int32_t *idx, int64_t n_seq,
                                 int64_t n_steps, int32_t n_experts, int32_t top_k, const int32_t *lags, int32_t n_lags,
                                 int32_t window, const double *coef, const double *loss_values, float *dlogits,
                                 void *workspace, size_t workspace_bytes, void *stream)
{
    remoe_status st = validate_trace(idx, n_seq, n_steps, top_k, n_experts);
    if (st != REMOE_OK) return st;
    if (n_lags < 0 || n_lags > 8 || (n_lags > 0 && !lags)) return fail(REMOE_E_INVALID_ARG, "n_lags %d outside 0..8 or lags is NULL", n_lags);
    for (int i = 0; i < n_lags; ++i)
        if (lags[i] < 1) return fail(REMOE_E_INVALID_ARG, "lag %d must be positive", lags[i]);
    if (window < 1) return fail(REMOE_E_INVALID_ARG, "window %d must be positive", window);
    if (!coef) return fail(REMOE_E_INVALID_ARG, "coef is NULL");
    for (int i = 0; i < 5; ++i)
        if (!(coef[i] == coef[i]) || coef[i] - coef[i] != 0.0) return fail(REMOE_E_INVALID_ARG, "coef[%d] is not finite", i);
    if (n_seq == 0 || n_steps == 0) return REMOE_OK;
    if (!probs || !probs_ref || !loss_values || !dlogits) return fail(REMOE_E_INVALID_ARG, "a required pointer is NULL");
    const size_t need = loss_backward_workspace_bytes(n_seq, n_steps, n_experts, window);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 7))
        return fail(REMOE_E_WORKSPACE, "remoe_loss_backward needs an 8-byte aligned workspace of %zu bytes", need);
    return launch_loss_backward(probs, probs_ref, idx, n_seq, n_steps, n_experts, top_k, lags, n_lags, window, coef,
                                loss_values, dlogits, workspace, static_cast<hipStream_t>(stream));
}

size_t remoe_gate_grad_workspace_bytes(int64_t n_tokens, int32_t n_experts, int32_t hidden)
{
    if (n_tokens < 0 || n_experts < 1 || hidden < 1) return 0;
    return gate_grad_workspace_bytes(n_tokens, n_experts, hidden);
}

remoe_status remoe_gate_grad(const float *dlogits, const void *x, int32_t x_dtype, int64_t n_tokens, int32_t n_experts,
                             int32_t hidden, float *dw, void *workspace, size_t workspace_bytes, void *stream)
{
    if (n_tokens < 0 || n_experts < 1 || n_experts > 128 || hidden < 1)
        return fail(REMOE_E_INVALID_ARG, "remoe_gate_grad: n_tokens %lld, n_experts %d (1..128), hidden %d", (long long)n_tokens,
                    n_experts, hidden);
    if (x_dtype != REMOE_F32 && x_dtype != REMOE_BF16) return fail(REMOE_E_INVALID_ARG, "x_dtype %d is neither REMOE_F32 nor REMOE_BF16", x_dtype);
    if (!dw || (n_tokens > 0 && (!dlogits || !x))) return fail(REMOE_E_INVALID_ARG, "a required pointer is NULL");
    const size_t need = gate_grad_workspace_bytes(n_tokens, n_experts, hidden);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255))
        return fail(REMOE_E_WORKSPACE, "remoe_gate_grad needs a 256-byte aligned workspace of %zu bytes", need);
    return launch_gate_grad(dlogits, x, x_dtype, n_tokens, n_experts, hidden, dw, workspace, static_cast<hipStream_t>(stream));
}

#pragma GCC visibility pop
}  // extern "C"
