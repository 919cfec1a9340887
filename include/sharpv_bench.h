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
 * "kv_cosine", "kv_mean", "kv_mask_scan", "kv_gather", "kv_gather_rope", "stream_copy", "stream_read",
 * "stream_read_slabs", "stream_gather_rows".
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

/* ------------------------------------------------------------------------------------------------
 * Floors of the pre-LLM stage's two memory-bound passes (not part of the method).
 *
 * sharpv_stream_read_slabs reads feats [n_frames, f, d] (f <= 208, elements of elem_bytes = 2 or 4 bytes,
 * row bytes a multiple of 16) in the order the fused statistics kernel reads it -- one workgroup per
 * compute unit walking a run of consecutive (256-column slab, frame) pairs, rows g, g+16, ... per thread,
 * one frame slab of loads in flight, the frame after a run read once more by the run before it -- and does
 * nothing with the data (`sink` as for sharpv_stream_read).  Timed as "stream_read_slabs".
 *
 * sharpv_stream_gather_rows copies n_idx rows of row_bytes bytes (a multiple of 16): dst row j = src row
 * idx[j] (device int32, each a valid row of src; dst must hold n_idx rows and not overlap src).  It is the
 * compaction of the token stream with the selection already made.  Timed as "stream_gather_rows".
 */
int sharpv_stream_read_slabs(const void* feats /* device */, int n_frames, int f, int d, int elem_bytes,
                             uint32_t* sink /* device */, void* stream);
int sharpv_stream_gather_rows(void* dst /* device */, const void* src /* device */, int row_bytes,
                              const int32_t* idx /* device */, int n_idx, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SHARPV_BENCH_H */
