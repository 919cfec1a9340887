// Host-side plumbing shared by the translation units of libsharpv: validated argument packs,
// workspace carving, and the hooks of the optional per-kernel event timing.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/sharpv.h"
#include "sharpv_device.hpp"

namespace sharpv {

constexpr int kGroup = 64;          // packed positions per 64-bit word of the keep mask
constexpr int kMaskWord = 16;       // packed positions per 16-bit word of the keep mask (one workgroup each)

// Packed-batch description of the intra-LLM stage (device arrays, or the scalar form when B == 1).
struct SeqDesc {
    const int32_t* seq_offsets;     // [B+1] or nullptr
    const int32_t* vis_start;       // [B]
    const int32_t* vis_offsets;     // [B+1]
    int B;
    int vis_start0;
    int n_vis;                      // rows of orig
    const int32_t* orig_row;        // [S] position -> row of orig (< 0 or >= n_vis: not a visual token), or nullptr:
                                    // then the visual tokens are the contiguous blocks described above
};

struct KvArgs {
    const void* hidden; const void* orig; const void* K; const void* V;
    int64_t kv_stride_h, kv_stride_s, out_stride_h;
    SeqDesc sd;
    int B, S, n_vis, d, H, D, dtype, kv_mode;
    float M;
    int32_t* out_idx; int32_t* out_count;
    void* K_out; void* V_out;
    float* out_cos; float* out_mean_cos;
    int32_t* out_orig_row;                          // orig_row of the kept positions (map form only), or nullptr
    const float* rope_cos; const float* rope_sin;   // [rope_len][D/2] each, or nullptr: plain copy of the K rows
    int rope_len, rope_layout;
    void* workspace;
    hipStream_t stream;
};

struct TokArgs {
    const void* feats;
    const int32_t* frame_offsets;   // device [B+1] or nullptr
    int B, n, f, d, dtype, mode, min_keep, measure;
    float w, K;
    int32_t* out_idx; int32_t* out_counts; int32_t* out_offsets;
    void* out_feats;
    float* out_scores; float* out_ratio;
    void* workspace;
    hipStream_t stream;
};

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

struct KvWorkspace {
    unsigned long long* group_mask;  // [n_groups] keep mask of 64 positions (written as 4 x 16 bits)
    int32_t* drop_seq;               // [B]
    float* cosv;                     // [n_vis]
    int32_t* word_base;              // [n_words + 1] kept positions before each 16-bit mask word (long sequences only)
    size_t bytes;
};

// Up to this many mask words every gather workgroup adds up the popcounts of the words before its own
// (cheap, and no extra launch); beyond it that would grow with the square of the sequence length, so a
// scan kernel writes the prefix once.
constexpr int kGatherSelfScanWords = 8192;

inline KvWorkspace carve_kv_workspace(void* base, int B, int S, int n_vis) {
    const size_t n_groups = ((size_t)S + kGroup - 1) / kGroup;
    char* p = (char*)base;
    size_t off = 0;
    KvWorkspace w;
    w.group_mask = (unsigned long long*)(p + off);  off += align_up(n_groups * 8);
    w.drop_seq = (int32_t*)(p + off);               off += align_up((size_t)B * 4);
    w.cosv = (float*)(p + off);                     off += align_up((size_t)n_vis * 4);
    const size_t n_words = ((size_t)S + kMaskWord - 1) / kMaskWord;
    w.word_base = (int32_t*)(p + off);              off += align_up((n_words + 1) * 4);
    w.bytes = off;
    return w;
}

// The fused mean + inner-product kernel keeps two packed frame slabs in registers: bf16 rows only, and at
// most 13 rows per thread (f <= 208).  Other shapes take the two-kernel path.
inline bool tok_uses_slab(int dtype, int f) { return dtype == SHARPV_BF16 && f <= 208; }
inline int tok_num_slabs(int d) { return (d + kBlockElems - 1) / kBlockElems; }

struct TokWorkspace {
    float* mean;        // [n, d]            frame means (two-kernel path only)
    float* aa;          // [nparts][n*f]     x.x       (per-slab shares on the fused path, nparts = slabs)
    float* am;          // [nparts][n*f]     x.mean
    float* ab;          // [nparts][n*f]     x.x_prev
    float* part_mm;     // [n][slabs]        mean.mean shares (fused path only)
    int32_t* local_idx; // [n*f]             kept rows of frame t at [t*f, t*f + count)
    int nparts;
    size_t bytes;
};

inline TokWorkspace carve_tok_workspace(void* base, int n, int f, int d, int dtype) {
    char* p = (char*)base;
    size_t off = 0;
    const size_t N = (size_t)n * f;
    const bool slab = tok_uses_slab(dtype, f);
    const int slabs = tok_num_slabs(d);
    TokWorkspace w;
    w.nparts = slab ? slabs : 1;
    w.mean = (float*)(p + off);         off += slab ? 0 : align_up((size_t)n * d * 4);
    w.aa = (float*)(p + off);           off += align_up((size_t)w.nparts * N * 4);
    w.am = (float*)(p + off);           off += align_up((size_t)w.nparts * N * 4);
    w.ab = (float*)(p + off);           off += align_up((size_t)w.nparts * N * 4);
    w.part_mm = (float*)(p + off);      off += slab ? align_up((size_t)n * slabs * 4) : 0;
    w.local_idx = (int32_t*)(p + off);  off += align_up(N * 4);
    w.bytes = off;
    return w;
}

// ---------------------------------------------------------------------------- event timing
enum KernelId { kFrameSlab = 0, kFrameMean, kTokenDots, kFrameSelect, kCountScan, kTokenGather,
                kKvCosine, kKvMean, kKvMaskScan, kKvGather, kKvGatherRope, kStreamCopy, kStreamRead, kStreamReadSlabs,
                kStreamGatherRows, kNumKernels };

// Hooks of the optional per-kernel event timing (sharpv_bench.hip).  While timing is off -- the normal
// state -- timing_begin is one atomic load and returns -1.
long long timing_begin(int kernel, hipStream_t st);      // reserves an event pair, records its start; -1: not timed
void timing_end(long long ticket, hipStream_t st);

struct TimedLaunch {
    long long ticket; hipStream_t st;
    TimedLaunch(int kernel, hipStream_t s) : ticket(timing_begin(kernel, s)), st(s) {}
    ~TimedLaunch() { timing_end(ticket, st); }
};

int launch_prune_tokens(const TokArgs& a);
int launch_prune_kv(const KvArgs& a);

}  // namespace sharpv
