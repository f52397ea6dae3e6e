/*
 * remoe_bench.h -- measurement aids of the benchmark drivers.  They are exported by the same
 * library as the entry points of remoe.h but are not part of the hot-path boundary: nothing on the
 * path needs them, and a deployment can ignore this header.
 */
#ifndef REMOE_BENCH_H
#define REMOE_BENCH_H

#include "remoe.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Optional per-kernel timing, for benchmarks.  While enabled, each kernel group an entry point
 * launches is bracketed by a pair of HIP events recorded on the caller's stream (a few
 * microseconds per pair; results are unaffected).  remoe_profile_read returns the summed elapsed
 * time and the number of launches of one kind since the last reset; the caller must have
 * synchronised the streams it used.  total_ms / launches are HOST pointers (either may be NULL).
 * Host calls; thread-safe; off by default.  remoe_profile_enable(1) creates the pool of events the
 * entry points draw from (4096 pairs, once); the entry points never create one, and a kernel
 * group that finds the pool empty goes unrecorded.
 */
typedef enum {
    REMOE_PROF_ROUTE = 0,          /* router GEMM + top-k + softmax                  */
    REMOE_PROF_PERMUTE = 1,        /* token -> expert sort and tile list             */
    REMOE_PROF_GATE_UP = 2,        /* routed experts: gate/up GEMM + SwiGLU          */
    REMOE_PROF_DOWN = 3,           /* routed experts: down GEMM x gate weight        */
    REMOE_PROF_SHARED_GATE_UP = 4, /* shared expert: gate/up GEMM + SwiGLU           */
    REMOE_PROF_SHARED_DOWN = 5,    /* shared expert: down GEMM                       */
    REMOE_PROF_COMBINE = 6,        /* sum of a token's rows                          */
    REMOE_PROF_TRACE_REUSE = 7,    /* adjacent-step overlap                          */
    REMOE_PROF_LRU = 8,            /* LRU cache misses                               */
    REMOE_PROF_DECODE = 9,         /* M = 1 decode kernel                            */
    REMOE_PROF_CACHE = 10,         /* cache_simulate (FIFO / LFU / Belady / LRU walk) */
    REMOE_PROF_KINDS = 11
} remoe_prof_kind;
remoe_status remoe_profile_enable(int32_t on);
remoe_status remoe_profile_read(int32_t kind, double *total_ms, int64_t *launches, int32_t reset);

/*
 * Measurement aid: a plain device-to-device copy of `bytes` bytes (a multiple of 16; dst and src
 * are 16-byte aligned device pointers that do not overlap), enqueued on `stream`.  It reads and
 * writes exactly `bytes` bytes of HBM, so the value a hardware byte counter reports for it gives
 * the factor by which that counter's readings for the other kernels are scaled.
 */
remoe_status remoe_copy_probe(void *dst, const void *src, size_t bytes, void *stream);

#ifdef __cplusplus
}
#endif

#endif /* REMOE_BENCH_H */
