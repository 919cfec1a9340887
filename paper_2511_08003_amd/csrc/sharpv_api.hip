// C ABI of libsharpv (declared in include/sharpv.h): argument validation on the host, then the
// launch sequences of sharpv_tokens.hip / sharpv_kv.hip.
#include <string.h>

#include <mutex>

#include "sharpv_kernels.hpp"

namespace sharpv {

static bool aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }

// ---------------------------------------------------------------------------- scratch of sharpv_prune_kv_static
// The intra-LLM stage's scratch (keep mask, per-sequence flags, cosines, mask prefix) for callers that may
// not allocate: a fixed array inside the library's code object instead of a caller workspace.  Every GPU
// the library runs on holds its own copy, at its own address, until the process ends.
constexpr int kStaticMaxS = SHARPV_STATIC_MAX_S;     // packed positions
constexpr int kStaticMaxB = SHARPV_STATIC_MAX_B;     // sequences
constexpr size_t kStaticScratchBytes = (size_t)5 << 18;   // 1.25 MiB >= the workspace of the largest admitted call
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Device address of `scratch` on the current device.  In host code the array's name is only a handle
// for hipGetSymbolAddress, never an address a kernel could use; the address is asked for once per
// device (with that device current) and kept.
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices] = {};

static int static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SHARPV_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
            (void)hipGetLastError();
            return SHARPV_ERR_DEVICE;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SHARPV_OK;
}

static int check_params(const sharpv_params* p) {
    if (p == nullptr) return SHARPV_ERR_NULL;
    if (p->struct_size != sizeof(sharpv_params)) return SHARPV_ERR_PARAM;
    if (p->dtype != SHARPV_F32 && p->dtype != SHARPV_BF16) return SHARPV_ERR_DTYPE;
    if (p->mode != 0 && p->mode != 1) return SHARPV_ERR_PARAM;
    if (p->kv_mode != 0 && p->kv_mode != 1) return SHARPV_ERR_PARAM;
    if (p->measure != SHARPV_DISSIM_EQ1 && p->measure != SHARPV_ONE_MINUS_COS) return SHARPV_ERR_PARAM;
    if (p->measure == SHARPV_ONE_MINUS_COS && p->mode != 1) return SHARPV_ERR_PARAM;   // pairing of Sec. 3.1
    if (p->min_keep < 0) return SHARPV_ERR_PARAM;
    if (!(p->w == p->w) || !(p->M == p->M) || !(p->K == p->K)) return SHARPV_ERR_PARAM;   // NaN
    return SHARPV_OK;
}

static int check_token_shape(int B, int n, int f, int d) {
    if (n < 1 || f < 1 || f > 1024 || d < 8 || d % 8 != 0 || d > 65536) return SHARPV_ERR_SHAPE;
    if (B < 1 || B > n) return SHARPV_ERR_SHAPE;
    if ((long long)n * f >= (1ll << 31)) return SHARPV_ERR_SHAPE;
    return SHARPV_OK;
}

static int check_kv_shape(int B, int S, int n_vis, int d) {
    if (S < 1 || n_vis < 0 || n_vis > S || d < 8 || d % 8 != 0 || d > 65536) return SHARPV_ERR_SHAPE;
    if (B < 1 || B > S) return SHARPV_ERR_SHAPE;
    return SHARPV_OK;
}

}  // namespace sharpv

using namespace sharpv;

extern "C" {

int sharpv_params_default(sharpv_params* p) {
    if (p == nullptr) return SHARPV_ERR_NULL;
    memset(p, 0, sizeof(*p));
    p->struct_size = (uint32_t)sizeof(sharpv_params);
    p->dtype = SHARPV_BF16;
    p->w = 1.0f;
    p->M = 0.2f;
    p->mode = 0;
    p->K = 1.6f;
    p->min_keep = 0;
    p->kv_mode = 0;
    p->measure = SHARPV_DISSIM_EQ1;
    return SHARPV_OK;
}

const char* sharpv_status_string(int status) {
    switch (status) {
        case SHARPV_OK: return "ok";
        case SHARPV_ERR_NULL: return "a required pointer is NULL";
        case SHARPV_ERR_SHAPE: return "a size is out of range or breaks an alignment rule";
        case SHARPV_ERR_DTYPE: return "unknown element type";
        case SHARPV_ERR_PARAM: return "invalid parameter block";
        case SHARPV_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case SHARPV_ERR_DEVICE: return "HIP call or kernel launch failed";
        case SHARPV_ERR_STATIC_LIMIT: return "sizes beyond what the library's built-in scratch holds";
        default: return "unknown status";
    }
}

int sharpv_version(void) { return 300; }   // 0.3.0: sharpv_params grew the `measure` field

size_t sharpv_prune_tokens_workspace(int n_frames, int f, int d, const sharpv_params* params) {
    if (check_params(params) != SHARPV_OK || check_token_shape(1, n_frames, f, d) != SHARPV_OK) return 0;
    return carve_tok_workspace(nullptr, n_frames, f, d, params->dtype).bytes;
}

int sharpv_prune_tokens(const void* feats, const int32_t* frame_offsets, int B, int n_frames, int f, int d,
                        const sharpv_params* params, int32_t* out_idx, int32_t* out_counts, int32_t* out_offsets,
                        void* out_feats, float* out_scores, float* out_ratio, void* workspace,
                        size_t workspace_bytes, void* stream) {
    int rc = check_params(params);
    if (rc != SHARPV_OK) return rc;
    if (feats == nullptr || out_idx == nullptr || out_counts == nullptr || out_offsets == nullptr ||
        out_feats == nullptr)
        return SHARPV_ERR_NULL;
    rc = check_token_shape(B, n_frames, f, d);
    if (rc != SHARPV_OK) return rc;
    if (frame_offsets == nullptr && B != 1) return SHARPV_ERR_NULL;
    if (params->min_keep > f) return SHARPV_ERR_PARAM;
    if (!aligned(feats, 16) || !aligned(out_feats, 16) || !aligned(out_idx, 4) || !aligned(out_counts, 4) ||
        !aligned(out_offsets, 4))
        return SHARPV_ERR_SHAPE;
    if (workspace == nullptr || !aligned(workspace, 256) ||
        workspace_bytes < carve_tok_workspace(nullptr, n_frames, f, d, params->dtype).bytes)
        return SHARPV_ERR_WORKSPACE;

    TokArgs a;
    a.feats = feats; a.frame_offsets = frame_offsets;
    a.B = B; a.n = n_frames; a.f = f; a.d = d;
    a.dtype = params->dtype; a.mode = params->mode; a.min_keep = params->min_keep; a.measure = params->measure;
    a.w = params->w; a.K = params->K;
    a.out_idx = out_idx; a.out_counts = out_counts; a.out_offsets = out_offsets;
    a.out_feats = out_feats; a.out_scores = out_scores; a.out_ratio = out_ratio;
    a.workspace = workspace; a.stream = (hipStream_t)stream;
    return launch_prune_tokens(a);
}

size_t sharpv_prune_kv_workspace(int B, int S, int n_vis, const sharpv_params* params) {
    if (check_params(params) != SHARPV_OK || check_kv_shape(B, S, n_vis, 8) != SHARPV_OK) return 0;
    return carve_kv_workspace(nullptr, B, S, n_vis).bytes;
}

}  // extern "C"

// Shared body of sharpv_prune_kv and sharpv_prune_kv_rope (rope_cos == nullptr: plain gather).
static int prune_kv_checked(const void* hidden, const void* orig, const void* K, const void* V, int64_t kv_stride_h,
                            int64_t kv_stride_s, const int32_t* seq_offsets, const int32_t* vis_start,
                            const int32_t* vis_offsets, int B, int S, int vis_start0, int n_vis, int d, int H, int D,
                            const sharpv_params* params, int32_t* out_idx, int32_t* out_count, void* K_out,
                            void* V_out, int64_t out_stride_h, float* out_cos, float* out_mean_cos,
                            const float* rope_cos, const float* rope_sin, int rope_len, int rope_layout,
                            const int32_t* orig_row, int32_t* out_orig_row,
                            void* workspace, size_t workspace_bytes, void* stream, bool validate_only = false) {
    int rc = check_params(params);
    if (rc != SHARPV_OK) return rc;
    if (hidden == nullptr || orig == nullptr || K == nullptr || V == nullptr || K_out == nullptr ||
        V_out == nullptr || out_idx == nullptr || out_count == nullptr)
        return SHARPV_ERR_NULL;
    rc = check_kv_shape(B, S, orig_row != nullptr ? 0 : n_vis, d);
    if (rc != SHARPV_OK) return rc;
    if (orig_row != nullptr) {                   // map form: only seq_offsets describes the batch
        if (B > 1 && seq_offsets == nullptr) return SHARPV_ERR_NULL;
    } else {
        const bool ragged = seq_offsets != nullptr || vis_start != nullptr || vis_offsets != nullptr;
        if (ragged && (seq_offsets == nullptr || vis_start == nullptr || vis_offsets == nullptr)) return SHARPV_ERR_NULL;
        if (!ragged) {
            if (B != 1) return SHARPV_ERR_NULL;
            if (vis_start0 < 0 || (long long)vis_start0 + n_vis > S) return SHARPV_ERR_SHAPE;
        }
    }
    const int64_t esz = params->dtype == SHARPV_F32 ? 4 : 2;
    if (H < 1 || D < 1 || (D * esz) % 16 != 0) return SHARPV_ERR_SHAPE;
    if (kv_stride_s < D || kv_stride_h < 1 || out_stride_h < D) return SHARPV_ERR_SHAPE;
    if ((kv_stride_s * esz) % 16 != 0 || (kv_stride_h * esz) % 16 != 0 || (out_stride_h * esz) % 16 != 0)
        return SHARPV_ERR_SHAPE;
    if (!aligned(hidden, 16) || !aligned(orig, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(K_out, 16) ||
        !aligned(V_out, 16) || !aligned(out_idx, 4) || !aligned(out_count, 4))
        return SHARPV_ERR_SHAPE;
    {   // the outputs are written while the inputs are still being read by other workgroups: no byte of
        // K_out / V_out (as far as a call that keeps everything would write) may lie inside K or V, nor
        // may the two outputs share bytes
        const uintptr_t in_span = (uintptr_t)(((int64_t)(H - 1) * kv_stride_h + (int64_t)(S - 1) * kv_stride_s + D) * esz);
        const uintptr_t out_span = (uintptr_t)(((int64_t)(H - 1) * out_stride_h + (int64_t)S * D) * esz);
        auto overlap = [](const void* a, uintptr_t na, const void* b, uintptr_t nb) {
            const uintptr_t pa = (uintptr_t)a, pb = (uintptr_t)b;
            return pa < pb + nb && pb < pa + na;
        };
        if (overlap(K_out, out_span, K, in_span) || overlap(K_out, out_span, V, in_span) ||
            overlap(V_out, out_span, K, in_span) || overlap(V_out, out_span, V, in_span) ||
            overlap(K_out, out_span, V_out, out_span))
            return SHARPV_ERR_SHAPE;
    }
    if (validate_only) return SHARPV_OK;         // everything but the workspace has been checked
    if (workspace == nullptr || !aligned(workspace, 256) ||
        workspace_bytes < carve_kv_workspace(nullptr, B, S, orig_row != nullptr ? S : n_vis).bytes)
        return SHARPV_ERR_WORKSPACE;

    KvArgs a;
    a.hidden = hidden; a.orig = orig; a.K = K; a.V = V;
    a.kv_stride_h = kv_stride_h; a.kv_stride_s = kv_stride_s; a.out_stride_h = out_stride_h;
    a.sd.seq_offsets = seq_offsets; a.sd.vis_start = vis_start; a.sd.vis_offsets = vis_offsets;
    a.sd.B = B; a.sd.vis_start0 = vis_start0; a.sd.n_vis = n_vis; a.sd.orig_row = orig_row;
    a.out_orig_row = out_orig_row;
    a.B = B; a.S = S; a.n_vis = n_vis; a.d = d; a.H = H; a.D = D;
    a.dtype = params->dtype; a.kv_mode = params->kv_mode; a.M = params->M;
    a.out_idx = out_idx; a.out_count = out_count; a.K_out = K_out; a.V_out = V_out;
    a.out_cos = out_cos; a.out_mean_cos = out_mean_cos;
    a.rope_cos = rope_cos; a.rope_sin = rope_sin; a.rope_len = rope_len; a.rope_layout = rope_layout;
    a.workspace = workspace; a.stream = (hipStream_t)stream;
    return launch_prune_kv(a);
}

extern "C" {

int sharpv_prune_kv(const void* hidden, const void* orig, const void* K, const void* V, int64_t kv_stride_h,
                    int64_t kv_stride_s, const int32_t* seq_offsets, const int32_t* vis_start,
                    const int32_t* vis_offsets, int B, int S, int vis_start0, int n_vis, int d, int H, int D,
                    int layer, const sharpv_params* params, int32_t* out_idx, int32_t* out_count, void* K_out,
                    void* V_out, int64_t out_stride_h, float* out_cos, float* out_mean_cos, void* workspace,
                    size_t workspace_bytes, void* stream) {
    (void)layer;
    return prune_kv_checked(hidden, orig, K, V, kv_stride_h, kv_stride_s, seq_offsets, vis_start, vis_offsets, B, S,
                            vis_start0, n_vis, d, H, D, params, out_idx, out_count, K_out, V_out, out_stride_h,
                            out_cos, out_mean_cos, nullptr, nullptr, 0, 0, nullptr, nullptr, workspace, workspace_bytes,
                            stream);
}

int sharpv_prune_kv_static(const void* hidden, const void* orig, const void* K, const void* V, int64_t kv_stride_h,
                           int64_t kv_stride_s, const int32_t* seq_offsets, const int32_t* vis_start,
                           const int32_t* vis_offsets, int B, int S, int vis_start0, int n_vis, int d, int H, int D,
                           int layer, const sharpv_params* params, int32_t* out_idx, int32_t* out_count, void* K_out,
                           void* V_out, int64_t out_stride_h, float* out_cos, float* out_mean_cos, void* stream) {
    (void)layer;
    // argument errors first (as in sharpv_prune_kv; they need no GPU), then the limits of the built-in
    // scratch, and only then its address
    const int rc_args = prune_kv_checked(hidden, orig, K, V, kv_stride_h, kv_stride_s, seq_offsets, vis_start,
                                         vis_offsets, B, S, vis_start0, n_vis, d, H, D, params, out_idx, out_count,
                                         K_out, V_out, out_stride_h, out_cos, out_mean_cos, nullptr, nullptr, 0, 0,
                                         nullptr, nullptr, /*workspace=*/nullptr, 0, stream, /*validate_only=*/true);
    if (rc_args != SHARPV_OK) return rc_args;
    if (S > kStaticMaxS || B > kStaticMaxB || carve_kv_workspace(nullptr, B, S, n_vis).bytes > kStaticScratchBytes)
        return SHARPV_ERR_STATIC_LIMIT;
    void* ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != SHARPV_OK) return rc;
    return prune_kv_checked(hidden, orig, K, V, kv_stride_h, kv_stride_s, seq_offsets, vis_start, vis_offsets, B, S,
                            vis_start0, n_vis, d, H, D, params, out_idx, out_count, K_out, V_out, out_stride_h,
                            out_cos, out_mean_cos, nullptr, nullptr, 0, 0, nullptr, nullptr, ws, kStaticScratchBytes,
                            stream);
}

int sharpv_prune_kv_rope(const void* hidden, const void* orig, const void* K, const void* V, int64_t kv_stride_h,
                         int64_t kv_stride_s, const int32_t* seq_offsets, const int32_t* vis_start,
                         const int32_t* vis_offsets, int B, int S, int vis_start0, int n_vis, int d, int H, int D,
                         int layer, const sharpv_params* params, int32_t* out_idx, int32_t* out_count, void* K_out,
                         void* V_out, int64_t out_stride_h, float* out_cos, float* out_mean_cos,
                         const float* rope_cos, const float* rope_sin, int rope_len, int rope_layout,
                         void* workspace, size_t workspace_bytes, void* stream) {
    (void)layer;
    if (rope_cos == nullptr || rope_sin == nullptr) return SHARPV_ERR_NULL;
    if (rope_layout != SHARPV_ROPE_HALF && rope_layout != SHARPV_ROPE_INTERLEAVED) return SHARPV_ERR_PARAM;
    if (params != nullptr && params->struct_size == sizeof(sharpv_params)) {
        // a half row must be whole 16-byte pieces, and the tables must reach the largest possible shift
        const int64_t esz = params->dtype == SHARPV_F32 ? 4 : 2;
        if (D < 2 || (D * esz) % 32 != 0 || rope_len < S) return SHARPV_ERR_SHAPE;
    }
    if (!aligned(rope_cos, 4) || !aligned(rope_sin, 4)) return SHARPV_ERR_SHAPE;
    return prune_kv_checked(hidden, orig, K, V, kv_stride_h, kv_stride_s, seq_offsets, vis_start, vis_offsets, B, S,
                            vis_start0, n_vis, d, H, D, params, out_idx, out_count, K_out, V_out, out_stride_h,
                            out_cos, out_mean_cos, rope_cos, rope_sin, rope_len, rope_layout, nullptr, nullptr,
                            workspace, workspace_bytes, stream);
}

size_t sharpv_prune_kv_carried_workspace(int B, int S, const sharpv_params* params) {
    return sharpv_prune_kv_workspace(B, S, S, params);
}

int sharpv_prune_kv_carried(const void* hidden, const void* orig, const int32_t* orig_row, const void* K, const void* V,
                            int64_t kv_stride_h, int64_t kv_stride_s, const int32_t* seq_offsets, int B, int S,
                            int n_orig, int d, int H, int D, int layer, const sharpv_params* params,
                            int32_t* out_idx, int32_t* out_count, void* K_out, void* V_out, int64_t out_stride_h,
                            int32_t* out_orig_row, float* out_cos, const float* rope_cos, const float* rope_sin,
                            int rope_len, int rope_layout, void* workspace, size_t workspace_bytes, void* stream) {
    (void)layer;
    if (orig_row == nullptr || out_orig_row == nullptr) return SHARPV_ERR_NULL;
    if (n_orig < 1) return SHARPV_ERR_SHAPE;
    if (params != nullptr && params->struct_size == sizeof(sharpv_params) && params->kv_mode != 0)
        return SHARPV_ERR_PARAM;                 // the per-sequence mean decision has no use for a map
    if (!aligned(orig_row, 4) || !aligned(out_orig_row, 4)) return SHARPV_ERR_SHAPE;
    const bool rope = rope_cos != nullptr || rope_sin != nullptr;
    if (rope) {
        if (rope_cos == nullptr || rope_sin == nullptr) return SHARPV_ERR_NULL;
        if (rope_layout != SHARPV_ROPE_HALF && rope_layout != SHARPV_ROPE_INTERLEAVED) return SHARPV_ERR_PARAM;
        if (params != nullptr && params->struct_size == sizeof(sharpv_params)) {
            const int64_t esz = params->dtype == SHARPV_F32 ? 4 : 2;
            if (D < 2 || (D * esz) % 32 != 0 || rope_len < S) return SHARPV_ERR_SHAPE;
        }
        if (!aligned(rope_cos, 4) || !aligned(rope_sin, 4)) return SHARPV_ERR_SHAPE;
    }
    // the shape checks take the number of rows of orig where the block form takes n_vis <= S; here a
    // shrunken sequence may well be shorter than orig, so S is checked on its own and n_orig rides along
    if (S < 1) return SHARPV_ERR_SHAPE;
    return prune_kv_checked(hidden, orig, K, V, kv_stride_h, kv_stride_s, seq_offsets, nullptr, nullptr, B, S, 0,
                            n_orig, d, H, D, params, out_idx, out_count, K_out, V_out, out_stride_h, out_cos, nullptr,
                            rope_cos, rope_sin, rope_len, rope_layout, orig_row, out_orig_row, workspace,
                            workspace_bytes, stream);
}

}  // extern "C"
