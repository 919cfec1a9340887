/*
 * sharpv.h -- C ABI of the SharpV pruning library for AMD MI355X (gfx950).
 *
 * SharpV (Sec. 3 of the paper) prunes a VideoLLM's visual tokens in two places:
 *
 *   sharpv_prune_tokens   pre-LLM stage, Sec. 3.1 "Information-Aware Visual Space Pruning":
 *                         spatial importance S (Eq.2) and temporal importance T (Eq.3) of every
 *                         token through the dissimilarity of Eq.1, score I = T + w S (Eq.4), a
 *                         per-frame retention ratio ||T_t||_2 / (2 sqrt f) (Eq.5; first frame of a
 *                         video from S, Eq.6), per-frame top-k by I, and the compacted token stream.
 *
 *   sharpv_prune_kv       intra-LLM stage, Sec. 3.2 "Information-Aware Memory Space Pruning":
 *                         cosine between each visual token's layer-l hidden state and its original
 *                         embedding, discard when it is below M (Eq.7), and the layer's K/V cache
 *                         gathered into a compacted cache.  Attention scores are never needed.
 *
 * Conventions (all entry points)
 *   - Every tensor pointer is CALLER-OWNED DEVICE MEMORY on the current HIP device unless it is
 *     marked "host".  The library never allocates, frees or keeps device memory; scratch space
 *     comes from the caller's workspace (query the size first; sharpv_prune_kv_static uses a fixed
 *     array of its own instead).  Base pointers of feats / hidden /
 *     orig / K / V / their outputs must be 16-byte aligned, the workspace 256-byte aligned.
 *   - Calls only ENQUEUE kernels on `stream` (a hipStream_t passed as void*; NULL = the null stream)
 *     and return without synchronising; they allocate nothing and record no memset, so a sequence
 *     of calls can be captured into a HIP graph and replayed (with the event timing of sharpv_bench.h off).
 *     Counts stay on the device, so output buffers are sized for the worst case (everything kept).
 *   - The return value is a sharpv_status.  Argument errors are found on the host before any
 *     launch and leave every output untouched; nothing throws or aborts across this boundary.
 *   - Inputs must be finite.  Scores are accumulated in float32 in a fixed order, so results do
 *     not depend on launch geometry and repeat bit for bit.
 *   - Overlapping calls that share a workspace race; calls on one stream are ordered.
 *   - The pruning calls keep no state of their own: host threads may call them at the same time, each
 *     with its own workspace and outputs.
 *   - Measurement aids (per-kernel event timing, plain streaming copy / read) are declared apart, in
 *     sharpv_bench.h; nothing in this header depends on them.
 */
#ifndef SHARPV_H
#define SHARPV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SHARPV_OK = 0,
    SHARPV_ERR_NULL = 1,        /* a required pointer is NULL */
    SHARPV_ERR_SHAPE = 2,       /* a size is out of range or violates an alignment rule */
    SHARPV_ERR_DTYPE = 3,       /* params->dtype is not a sharpv_dtype */
    SHARPV_ERR_PARAM = 4,       /* params->struct_size / mode / kv_mode / min_keep / measure invalid */
    SHARPV_ERR_WORKSPACE = 5,   /* workspace NULL, misaligned or too small */
    SHARPV_ERR_DEVICE = 6,      /* a HIP call or kernel launch failed */
    SHARPV_ERR_STATIC_LIMIT = 7 /* sharpv_prune_kv_static only: S or B beyond the built-in scratch */
} sharpv_status;

typedef enum { SHARPV_F32 = 0, SHARPV_BF16 = 1 } sharpv_dtype;

/* How far apart two token vectors are, for S (Eq.2) and T (Eq.3).  Sec. 3.1 (Dissimilarity
 * Computation Module) uses Eq.1 throughout and names one stand-in, the rescaled cosine 1 - cos,
 * to go with a fixed threshold K: SHARPV_ONE_MINUS_COS is accepted only with mode == 1. */
typedef enum { SHARPV_DISSIM_EQ1 = 0, SHARPV_ONE_MINUS_COS = 1 } sharpv_measure;

/* Hyper-parameters (Sec. 4.1, Implementation Details: adaptive setting M = 0.2, w = 1; the
 * semi-adaptive setting adds a fixed threshold K = 1.6). */
typedef struct sharpv_params {
    uint32_t struct_size;   /* = sizeof(sharpv_params); checked */
    int32_t  dtype;         /* sharpv_dtype of feats / hidden / orig / K / V */
    float    w;             /* Eq.4 weight of the spatial importance */
    float    M;             /* Eq.7 degradation threshold */
    int32_t  mode;          /* 0: adaptive retention ratio + per-frame top-k (Eq.5/6);
                               1: keep token iff I >= K (manual threshold) */
    float    K;             /* manual threshold, used when mode == 1 */
    int32_t  min_keep;      /* lower clamp of the per-frame kept count (mode 0), 0 <= min_keep <= f */
    int32_t  kv_mode;       /* 0: Eq.7 per visual token;
                               1: Eq.7 on the mean cosine of a sequence's visual tokens (all or none) */
    int32_t  measure;       /* sharpv_measure for S and T; SHARPV_ONE_MINUS_COS needs mode == 1 */
} sharpv_params;

/* Fills *p with the paper's defaults (bf16, w=1, M=0.2, mode 0, K=1.6, min_keep 0, kv_mode 0, Eq.1). */
int sharpv_params_default(sharpv_params* p /* host */);

/* Static, NUL-terminated description of a status code. */
const char* sharpv_status_string(int status);

/* Library version: major*10000 + minor*100 + patch. */
int sharpv_version(void);

/* ------------------------------------------------------------------------------------------------
 * Pre-LLM stage (Sec. 3.1, Eq.1-6).
 *
 * feats is a packed batch of B videos: [n_frames, f, d] row-major, one token per row, where n_frames
 * is the total over the batch and video b owns frames [frame_offsets[b], frame_offsets[b+1]).  The
 * first frame of every video takes T := S (Eq.6); frames never look across a video boundary.
 *
 * Limits: 1 <= f <= 1024, d a positive multiple of 8 up to 65536, n_frames*f < 2^31, 1 <= B <= n_frames.
 */
size_t sharpv_prune_tokens_workspace(int n_frames, int f, int d, const sharpv_params* params /* host */);

int sharpv_prune_tokens(
    const void*    feats,          /* device [n_frames, f, d], params->dtype */
    const int32_t* frame_offsets,  /* device [B+1] ascending, [0]=0, [B]=n_frames; NULL => one video (B must be 1) */
    int B, int n_frames, int f, int d,
    const sharpv_params* params,   /* host */
    int32_t* out_idx,              /* device, capacity n_frames*f: kept global row indices t*f+i, ascending */
    int32_t* out_counts,           /* device [n_frames]: kept tokens per frame */
    int32_t* out_offsets,          /* device [n_frames+1]: exclusive scan of out_counts; last = total kept */
    void*    out_feats,            /* device, capacity n_frames*f*d: rows [0, total kept) = feats[out_idx[j]] */
    float*   out_scores,           /* device [n_frames*f] I (Eq.4), or NULL */
    float*   out_ratio,            /* device [n_frames] retention ratio (Eq.5/6), or NULL */
    void* workspace, size_t workspace_bytes,
    void* stream);

/* ------------------------------------------------------------------------------------------------
 * Intra-LLM stage for one decoder layer (Sec. 3.2, Eq.7).
 *
 * hidden is the layer's hidden-state matrix of a packed batch of B sequences, [S, d]; sequence b owns
 * packed positions [seq_offsets[b], seq_offsets[b+1]), its visual block starts vis_start[b] positions
 * into the sequence and its original embeddings are rows [vis_offsets[b], vis_offsets[b+1]) of orig.
 * With B == 1 the three arrays may be NULL and the scalars vis_start0 / n_vis describe the only
 * sequence.  Positions outside the visual blocks (system and instruction tokens) are always kept.
 *
 * K and V are [H, S, D] with element strides kv_stride_h (between heads) and kv_stride_s (between
 * positions), D contiguous.  K_out / V_out receive [H, S_kept, D] with head stride out_stride_h
 * (>= S*D is always enough) and position stride D; the byte ranges they may be written in
 * ([base, base + (H-1)*out_stride_h + S*D) elements) must not overlap the ranges K / V span nor each
 * other (checked on the host: SHARPV_ERR_SHAPE).
 *
 * Limits: d a positive multiple of 8 up to 65536; D*sizeof(element) and all strides*sizeof(element)
 * multiples of 16; 1 <= B <= S < 2^31; 0 <= n_vis <= S.
 */
size_t sharpv_prune_kv_workspace(int B, int S, int n_vis, const sharpv_params* params /* host */);

int sharpv_prune_kv(
    const void* hidden,            /* device [S, d] */
    const void* orig,              /* device [n_vis, d] */
    const void* K, const void* V,  /* device [H, S, D] (strided) */
    int64_t kv_stride_h, int64_t kv_stride_s,
    const int32_t* seq_offsets,    /* device [B+1] or NULL (B == 1) */
    const int32_t* vis_start,      /* device [B]   or NULL (B == 1) */
    const int32_t* vis_offsets,    /* device [B+1] or NULL (B == 1) */
    int B, int S, int vis_start0, int n_vis, int d, int H, int D,
    int layer,                     /* carried for the caller's bookkeeping; does not change the result */
    const sharpv_params* params,   /* host */
    int32_t* out_idx,              /* device, capacity S: kept packed positions, ascending */
    int32_t* out_count,            /* device [B]: kept positions per sequence */
    void* K_out, void* V_out,      /* device [H, <=S, D], head stride out_stride_h */
    int64_t out_stride_h,
    float* out_cos,                /* device [n_vis] cosine per visual token, or NULL */
    float* out_mean_cos,           /* device [B] mean cosine per sequence, or NULL */
    void* workspace, size_t workspace_bytes,
    void* stream);

/* ------------------------------------------------------------------------------------------------
 * sharpv_prune_kv for callers that cannot allocate or carry a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.
 *
 * Same arguments (without the workspace), decisions and outputs as sharpv_prune_kv.  The scratch memory
 * of its kernels (keep mask, per-sequence flags, cosines, mask prefix) is a fixed 1.25 MiB array inside
 * the library's code object; each GPU the library runs on holds its own copy until the process ends.
 * The call allocates nothing and frees nothing.  Its first call on a device looks the array's address up
 * (hipGetSymbolAddress, once per device, with that device current); make that first call outside a
 * stream capture.
 *
 * Limits beyond those of sharpv_prune_kv: S <= SHARPV_STATIC_MAX_S, B <= SHARPV_STATIC_MAX_B; larger calls
 * return SHARPV_ERR_STATIC_LIMIT and touch nothing.  All calls on one GPU share that GPU's array, which
 * keeps the previous call's contents (the kernels overwrite every word they later read, so nothing has
 * to be cleared): calls that overlap in time on one GPU -- other streams, other host threads -- race.
 * Calls on one stream are ordered.
 */
#define SHARPV_STATIC_MAX_S 262144
#define SHARPV_STATIC_MAX_B 256

int sharpv_prune_kv_static(
    const void* hidden, const void* orig, const void* K, const void* V,
    int64_t kv_stride_h, int64_t kv_stride_s,
    const int32_t* seq_offsets, const int32_t* vis_start, const int32_t* vis_offsets,
    int B, int S, int vis_start0, int n_vis, int d, int H, int D, int layer,
    const sharpv_params* params,   /* host */
    int32_t* out_idx, int32_t* out_count,
    void* K_out, void* V_out, int64_t out_stride_h,
    float* out_cos, float* out_mean_cos,
    void* stream);

/* ------------------------------------------------------------------------------------------------
 * Intra-LLM stage with positional re-encoding (Sec. 4.1, Implementation Details: the positional
 * embedding is re-encoded during intra-LLM pruning).
 *
 * Same decisions, outputs and limits as sharpv_prune_kv, except that every kept K row leaves with the
 * rotary embedding of its NEW place: a row that sat at position p of its sequence and becomes that
 * sequence's j-th kept row is turned back by delta = p - j steps.  The model's rotary convention stays
 * with the caller: rope_cos / rope_sin are device tables [rope_len][D/2] of float32 whose row `delta`
 * holds cos / sin of delta * theta_i (i-th frequency), and rope_layout says which elements form pair i
 * (SHARPV_ROPE_HALF: i and i + D/2; SHARPV_ROPE_INTERLEAVED: 2i and 2i+1).  Per pair (x, y), in float32:
 *     x' = fma(x, c, y*s),  y' = fma(y, c, -(x*s)),   rounded once to params->dtype.
 * V rows are copied unchanged.  Extra limits: D*sizeof(element) a multiple of 32 (a half row is whole
 * 16-byte pieces), rope_len >= S (no shift can be larger), tables 4-byte aligned and caller-owned.
 */
typedef enum { SHARPV_ROPE_HALF = 0, SHARPV_ROPE_INTERLEAVED = 1 } sharpv_rope_layout;

int sharpv_prune_kv_rope(
    const void* hidden, const void* orig, const void* K, const void* V,
    int64_t kv_stride_h, int64_t kv_stride_s,
    const int32_t* seq_offsets, const int32_t* vis_start, const int32_t* vis_offsets,
    int B, int S, int vis_start0, int n_vis, int d, int H, int D, int layer,
    const sharpv_params* params,   /* host */
    int32_t* out_idx, int32_t* out_count,
    void* K_out, void* V_out, int64_t out_stride_h,
    float* out_cos, float* out_mean_cos,
    const float* rope_cos,         /* device [rope_len, D/2] */
    const float* rope_sin,         /* device [rope_len, D/2] */
    int rope_len, int rope_layout,
    void* workspace, size_t workspace_bytes,   /* sized by sharpv_prune_kv_workspace */
    void* stream);

/* ------------------------------------------------------------------------------------------------
 * Intra-LLM stage carried from layer to layer (Sec. 3.2, Degradation-Aware Pruning: what a layer
 * discards does not propagate further, so the layers after it work on the survivors only).
 *
 * hidden [S, d] and K / V [H, S, D] hold the positions still alive at this layer; orig_row[s] is the row
 * of orig [n_orig, d] that position s started from, or -1 for a system / instruction position (any value
 * outside [0, n_orig) counts as -1).  A visual position is discarded iff the cosine between its hidden
 * state and that row is below M (Eq.7, per token: params->kv_mode must be 0); the others are always kept.
 * Beside the outputs of sharpv_prune_kv it writes out_orig_row[j] = orig_row[out_idx[j]], which is the
 * orig_row of the next layer's (shorter) sequence; out_cos, if given, is indexed by POSITION ([S], written
 * at visual positions only).  With rope_cos / rope_sin non-NULL the kept K rows are re-encoded exactly as
 * by sharpv_prune_kv_rope (positions counted inside the current, already shortened sequences).
 * seq_offsets may be NULL when B == 1.  Workspace: sharpv_prune_kv_carried_workspace(B, S, params).
 */
size_t sharpv_prune_kv_carried_workspace(int B, int S, const sharpv_params* params /* host */);

int sharpv_prune_kv_carried(
    const void* hidden,            /* device [S, d] */
    const void* orig,              /* device [n_orig, d] */
    const int32_t* orig_row,       /* device [S] */
    const void* K, const void* V,  /* device [H, S, D] (strided) */
    int64_t kv_stride_h, int64_t kv_stride_s,
    const int32_t* seq_offsets,    /* device [B+1] or NULL (B == 1) */
    int B, int S, int n_orig, int d, int H, int D, int layer,
    const sharpv_params* params,   /* host */
    int32_t* out_idx, int32_t* out_count,
    void* K_out, void* V_out, int64_t out_stride_h,
    int32_t* out_orig_row,         /* device, capacity S */
    float* out_cos,                /* device [S] or NULL */
    const float* rope_cos, const float* rope_sin, int rope_len, int rope_layout,   /* both NULL: K rows copied as they are */
    void* workspace, size_t workspace_bytes,
    void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SHARPV_H */
