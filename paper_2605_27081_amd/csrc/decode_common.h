// Device helpers shared by the two M = 1 decode kernels (layer-chained and layer-pipelined):
// cross-workgroup exchange through agent-scope atomics, the flag-array grid barrier with bounded
// waits, the 16-byte dot product, and the online routing-trace statistics (Eq. 1 overlap, App. E.2
// LRU misses).  The templates take the kernel's argument struct, which provides the fields they name.
#pragma once

#include "common.h"

namespace remoe {

namespace {

constexpr int DEC_THREADS = 512;        // both kernels run 8 wavefronts per workgroup
constexpr int DEC_MAX_CAPS = 4;
constexpr int DEC_MAX_LAYERS = 64;      // trace state of all layers is kept in LDS
constexpr int DEC_MAX_GRID = 1024;      // workgroups the flag barrier can hold
constexpr int DEC_FLAG_BYTES = 256 + DEC_MAX_GRID * 4;   // abort flag at byte 128, barrier flags from byte 256
constexpr int DEC_SEG = 256;            // router row segment per wavefront (floats)
constexpr int DEC_RING = 4;             // layer-steps whose exchanged values are kept apart (pipelined kernel)

constexpr int DEC_GROUPS = 8;           // workgroup groups of the pipelined kernel, each with its own rings

// Workspace: flags, then per group DEC_RING slots of tagged partial logits, then per group DEC_RING
// slots of tagged SwiGLU activations.  The chained kernel uses the first slot of each region.
struct DecodeWsLayout {
    size_t logit_off, h_off, total;
    int n_logit, n_h;                   // 8-byte words per ring slot
};
inline DecodeWsLayout decode_ws_layout(int H, int N, int I, int K)
{
    DecodeWsLayout l;
    l.n_logit = N * (H / DEC_SEG);
    l.n_h = K * I > DEC_MAX_GRID * 8 ? K * I : DEC_MAX_GRID * 8;   // chained: K*I floats; pipelined: one word per wavefront
    l.logit_off = DEC_FLAG_BYTES;
    l.h_off = l.logit_off + align_up(sizeof(unsigned long long) * (size_t)DEC_GROUPS * DEC_RING * l.n_logit, 256);
    l.total = l.h_off + align_up(sizeof(unsigned long long) * (size_t)DEC_GROUPS * DEC_RING * l.n_h, 256);
    return l;
}

// Load through a pointer that is known to point to device (global) memory.  Weight pointers come out
// of a table in memory, so the compiler cannot tell their address space and would emit flat loads:
// those need a 64-bit address register pair per lane and also count as LDS traffic, which makes every
// LDS wait a wait for the weight stream.
template <class T>
__device__ __forceinline__ T load_global(const void *p)
{
    return *(const __attribute__((address_space(1))) T *)p;
}

// The same as a non-temporal load, for the expert weights: every byte of them is read once per step
// and the next step's copy is tens of gigabytes away, so keeping them in the caches only pushes out
// what is reused (x, the exchange words).  Measured on the Qwen3-shaped stack: 13.15 -> 11.7 us per
// layer-step.
template <class T>
__device__ __forceinline__ T load_global_stream(const void *p)
{
    return __builtin_nontemporal_load((const __attribute__((address_space(1))) T *)p);
}

// Entry idx (the same for every lane) of the launch's weight-pointer table, read with a scalar
// load.  The host writes the table before the launch and no kernel ever does, so the constant
// address space is safe; a vector load here returns the pointer in the same in-order queue as the
// weight stream, and the wavefront would wait for every weight load in flight before using it.
__device__ __forceinline__ const void *table_ptr(const void *const *table, int idx)
{
    typedef const unsigned long long __attribute__((address_space(4))) *const_u64_ptr;
    return reinterpret_cast<const void *>(*(const_u64_ptr)(uintptr_t)(table + idx));
}

// Dot product of 8 bf16 pairs (two 16-byte registers) added to acc: four v_dot2c_f32_bf16 (exact
// products, fp32 accumulation).  Written as assembly because the compiler's builtin for this
// instruction picked the same source registers for all four elements of a 16-byte vector.  The
// compiler therefore does not know these are dot instructions either, so the idle states the
// hardware requires before another kind of vector instruction reads a dot result (three) are part
// of the block.
__device__ __forceinline__ float dot8_bf16(const u32x4_t w, const u32x4_t x, float acc)
{
#if defined(__HIP_DEVICE_COMPILE__)
    asm("v_dot2c_f32_bf16 %0, %1, %5\n\t"
        "v_dot2c_f32_bf16 %0, %2, %6\n\t"
        "v_dot2c_f32_bf16 %0, %3, %7\n\t"
        "v_dot2c_f32_bf16 %0, %4, %8\n\t"
        "s_nop 2"
        : "+v"(acc)
        : "v"(w.x), "v"(w.y), "v"(w.z), "v"(w.w), "v"(x.x), "v"(x.y), "v"(x.z), "v"(x.w));
#else
    (void)w;
    (void)x;
#endif
    return acc;
}

// Data that crosses workgroups inside the kernel (partial logits, SwiGLU activations) is written and
// read with agent-scope relaxed atomics: such stores write through the per-XCD L2 and such loads
// bypass it, so no cache write-back or invalidate is needed at the grid barriers.
__device__ __forceinline__ void put_shared(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float get_shared(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// A value and the number of the phase that produced it, as one 8-byte word.
__device__ __forceinline__ void put_tagged(unsigned long long *p, float v, uint32_t tag)
{
    __hip_atomic_store(p, ((unsigned long long)tag << 32) | __float_as_uint(v), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}

// Grid-wide barrier without read-modify-write traffic: workgroup b publishes the number of the phase
// it has finished in flags[b]; wavefront 0 of every workgroup polls all flags (each lane a few of
// them) until none is behind.  The workgroup barrier in front makes every wavefront wait for its own
// stores first (they are complete at agent scope then).  Returns false when the grid is aborting.
template <class Args>
__device__ __forceinline__ bool grid_barrier(const Args &a, uint32_t phase, int *lds_flag)
{
    __syncthreads();
    if (threadIdx.x < 64) {
        const int lane = threadIdx.x;
        const int G = gridDim.x;
        if (lane == 0) __hip_atomic_store(&a.bar[blockIdx.x], phase, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int ok = 1;
        unsigned long long t0 = 0;
        bool timing = false;
        for (;;) {
            // one memory round trip per poll: the abort flag travels with the flags
            const uint32_t ab = __hip_atomic_load(a.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            bool behind = false;
            for (int q = lane; q < G; q += 64)
                behind |= __hip_atomic_load(&a.bar[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < phase;
            if (!__any(behind)) break;
            if (!timing) { t0 = wall_clock64(); timing = true; }
            if (ab) { ok = 0; break; }
            if (wall_clock64() - t0 > a.spin_limit) {
                __hip_atomic_store(a.abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ok = 0;
                break;
            }
        }
        if (lane == 0) *lds_flag = ok;
    }
    __syncthreads();
    return *lds_flag != 0;
}

// Rendezvous on tagged values: every thread polls its share of the n words until all of them carry
// `tag`, leaving the values in LDS.  Returns false when the grid is aborting.
template <class Args>
__device__ __forceinline__ bool gather_tagged(const Args &a, float *dst, int n, uint32_t tag, int *lds_flag)
{
    unsigned long long t0 = 0;
    bool timing = false;
    for (;;) {
        uint32_t ab = 0;
        if (threadIdx.x == 0) ab = __hip_atomic_load(a.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        bool behind = false;
        for (int q = threadIdx.x; q < n; q += DEC_THREADS) {
            const unsigned long long w = __hip_atomic_load(&a.logit_part[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if ((uint32_t)(w >> 32) == tag) dst[q] = __uint_as_float((uint32_t)w);
            else behind = true;
        }
        if (threadIdx.x == 0) {
            int ok = 1;
            if (ab) ok = 0;
            if (!timing) { t0 = wall_clock64(); timing = true; }
            else if (wall_clock64() - t0 > a.spin_limit) {
                __hip_atomic_store(a.abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ok = 0;
            }
            *lds_flag = ok;
        }
        const int any_behind = __syncthreads_or(behind ? 1 : 0);
        if (!*lds_flag) return false;
        if (!any_behind) return true;
        __syncthreads();      // lds_flag is rewritten in the next round
    }
}

__device__ __forceinline__ float dot8(const u32x4_t w, const float *xv, float acc)
{
    acc = fmaf(__uint_as_float(w.x << 16), xv[0], acc);
    acc = fmaf(__uint_as_float(w.x & 0xFFFF0000u), xv[1], acc);
    acc = fmaf(__uint_as_float(w.y << 16), xv[2], acc);
    acc = fmaf(__uint_as_float(w.y & 0xFFFF0000u), xv[3], acc);
    acc = fmaf(__uint_as_float(w.z << 16), xv[4], acc);
    acc = fmaf(__uint_as_float(w.z & 0xFFFF0000u), xv[5], acc);
    acc = fmaf(__uint_as_float(w.w << 16), xv[6], acc);
    acc = fmaf(__uint_as_float(w.w & 0xFFFF0000u), xv[7], acc);
    return acc;
}

// Per-layer trace state of the one wavefront that keeps the statistics; it lives in LDS for the whole
// kernel and is loaded from / stored to device memory at the kernel's ends.
struct TraceLds {
    uint32_t last[DEC_MAX_LAYERS][128];                 // (step of last use) + 1, 0 = never
    unsigned long long sum_ov[DEC_MAX_LAYERS];
    unsigned long long tot[DEC_MAX_CAPS][DEC_MAX_LAYERS];
};

// Online overlap and LRU misses of one layer-step (one wavefront).  Lane l owns experts l, l + 64.
template <class Args>
__device__ __forceinline__ void online_trace_stats(const Args &a, TraceLds &ts, int layer, int64_t g,
                                                   const int *sel_e, int lane)
{
    const int N = a.N, K = a.K;
    const uint32_t last0 = ts.last[layer][lane], last1 = ts.last[layer][lane + 64];
    bool req0 = false, req1 = false;
    for (int j = 0; j < K; ++j) {
        const int e = sel_e[j];          // LDS broadcast
        req0 |= (e == lane);
        req1 |= (e == lane + 64);
    }
    req0 &= lane < N;
    req1 &= lane + 64 < N;
    // experts of the previous step carry last == g (they were stamped (g - 1) + 1)
    const int ov = (g > 0) ? __popcll(__ballot(req0 && last0 == (uint32_t)g)) +
                                 __popcll(__ballot(req1 && last1 == (uint32_t)g))
                           : 0;
    const uint32_t key0 = last0 ? ((last0 << 7) | (uint32_t)lane) : 0u;
    const uint32_t key1 = last1 ? ((last1 << 7) | (uint32_t)(lane + 64)) : 0u;
    unsigned long long m0 = __ballot(req0), m1 = __ballot(req1);
    const int n_unique = __popcll(m0) + __popcll(m1);
    int hits[DEC_MAX_CAPS] = {0, 0, 0, 0};
    while (m0 | m1) {
        uint32_t ke;
        if (m0) {
            const int b = __ffsll((long long)m0) - 1;
            m0 &= m0 - 1;
            ke = __shfl(key0, b, 64);
        } else {
            const int b = __ffsll((long long)m1) - 1;
            m1 &= m1 - 1;
            ke = __shfl(key1, b, 64);
        }
        const int above = __popcll(__ballot(key0 > ke)) + __popcll(__ballot(key1 > ke));
#pragma unroll
        for (int c = 0; c < DEC_MAX_CAPS; ++c) hits[c] += (c < a.n_caps && ke != 0u && above < a.caps[c]);
    }
    if (req0) ts.last[layer][lane] = (uint32_t)(g + 1);
    if (req1) ts.last[layer][lane + 64] = (uint32_t)(g + 1);
    if (lane == 0) {
        a.out_overlap[(int64_t)layer * a.steps_total + g] = (uint8_t)ov;
        ts.sum_ov[layer] += (unsigned long long)ov;
        for (int c = 0; c < a.n_caps; ++c) {
            const int miss = n_unique - hits[c];
            a.out_miss[((int64_t)c * a.n_layers + layer) * a.steps_total + g] = (uint8_t)miss;
            ts.tot[c][layer] += (unsigned long long)miss;
        }
    }
}

}  // namespace

}  // namespace remoe
