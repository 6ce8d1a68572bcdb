/*
 * gkv_bench.h - measurement aids of libgkv.so for benchmarks.  Not part of the method: kernel
 * timing hooks and a streaming-read probe that the benchmark reports next to the kernels' rates.
 */
#ifndef GKV_BENCH_H
#define GKV_BENCH_H

#include "gkv.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Kernel timing.  While enabled, each kernel launch is bracketed
 * by HIP events on the launch stream that record the kernel's own begin and
 * end; gkv_profile_read synchronises those events and returns the total
 * milliseconds and launch count of one kernel class since the last reset.
 */
typedef enum {
  GKV_K_ATTEND = 0, GKV_K_SCORE = 1, GKV_K_GLOBAL = 2, GKV_K_TOPK = 3, GKV_K_COMPACT = 4,
  GKV_K_REDUNDANCY = 5, GKV_K_COUNT = 6
} gkv_kernel_id;
gkv_status gkv_profile_enable(gkv_ctx* ctx, int32_t on);
gkv_status gkv_profile_read(gkv_ctx* ctx, int32_t kernel_id, double* total_ms, int64_t* launches);
gkv_status gkv_profile_reset(gkv_ctx* ctx);

/*
 * Read-bandwidth probe: the memory access pattern of the matrix-core decode kernel with nothing
 * else.  One workgroup of 4 wavefronts per unit streams rows [0, rows) of that unit's K block
 * (tiled format: 1 KiB contiguous per load, ordinary loads) and V block (256-byte rows,
 * non-temporal loads) of a bf16, d = 128 cache laid out [units, capacity, 128], folds the data
 * into a word it practically never stores, and does no arithmetic, softmax, merge or output.
 * Timing it on the benchmark's own cache gives the rate the memory system grants this pattern:
 * the ceiling the decode kernel is compared with.  rows must be a multiple of 16, at most
 * capacity; `sink` is 4 bytes of device memory.
 */
gkv_status gkv_probe_attend_read(const void* K, const void* V, int32_t units, int32_t capacity,
                                 int32_t rows, void* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* GKV_BENCH_H */
