/*
 * sharpv_bench.h -- measurement aids of libsharpv, apart from the method's entry points (sharpv.h).
 *
 * Nothing here belongs to SharpV's two pruning stages: these calls exist so that a benchmark can time the
 * library's kernels one by one on the launch stream, and set them against what the device's memory system
 * delivers for a plain read and a plain copy.  Status codes are those of sharpv.h.
 */
#ifndef SHARPV_BENCH_H
#define SHARPV_BENCH_H

#include <stddef.h>
#include <stdint.h>

#include "sharpv.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ------------------------------------------------------------------------------------------------
 * Per-kernel timing with HIP events on the launch stream (for benchmarks; off by default).
 * While enabled, every kernel launch of the two entry points is bracketed by a pair of events
 * taken from a pool of `max_launches` pairs (launches beyond the pool go untimed).
 * sharpv_timing_read synchronises on the recorded events and returns, for the kernel with the
 * given name, the number of timed launches and their summed duration in milliseconds.
 * Kernel names: "frame_slab", "frame_mean", "token_dots", "frame_select", "count_scan", "token_gather",
 * "kv_cosine", "kv_mean", "kv_mask_scan", "kv_gather", "kv_gather_rope", "stream_copy", "stream_read".
 * The pool is process-wide and guarded by a lock: host threads may launch while timing is on (each launch
 * keeps its own pair), and a launch that straddles enable / disable is dropped.  One device at a time.
 */
int sharpv_timing_enable(int max_launches);     /* creates the pool; resets earlier records */
int sharpv_timing_disable(void);                /* destroys the pool */
int sharpv_timing_read(const char* kernel_name, int* n_launches /* host */, double* total_ms /* host */);

/* ------------------------------------------------------------------------------------------------
 * Measurement aids (not part of the method): a plain streaming copy and a plain streaming read of
 * `bytes` bytes (a multiple of 16; 16-byte aligned device pointers), enqueued on `stream`.  They give
 * the practical HBM ceiling of the device next to the pruning kernels, and a copy of known size
 * against which hardware byte counters can be scaled.  sharpv_stream_read writes one 4-byte word to
 * `sink` (device) only if the data XORs to a magic value, i.e. practically never.
 * Timed under the kernel names "stream_copy" and "stream_read".
 */
int sharpv_stream_copy(void* dst /* device */, const void* src /* device */, size_t bytes, void* stream);
int sharpv_stream_read(const void* src /* device */, size_t bytes, uint32_t* sink /* device */, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SHARPV_BENCH_H */
