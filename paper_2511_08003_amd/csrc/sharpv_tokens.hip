// Pre-LLM stage (Sec. 3.1, Eq.1-6): frame means, per-token inner products, dissimilarities and
// scores, per-frame retention ratio and top-k, and the compaction of the token stream.
//
// Kernels
//   frame_mean    workgroup = (frame, 256-column slab), 32 row classes x 32 lanes: row i goes to
//                 class i % 32, each class adds its rows in ascending order, the 32 classes are
//                 reduced by a halving tree in LDS, divided by f.  Eq.2's average representation.
//   token_dots    one wavefront per token row: x.x, x.mean_t and x.x_prev in the fixed order of
//                 sharpv_device.hpp (the row, its predecessor in the previous frame and the frame
//                 mean are streamed with 16-byte loads).
//   frame_select  one workgroup per frame, one thread per token: Eq.1-4 from the stored inner
//                 products, Eq.5/6 retention ratio and kept count, rank of every token by counting
//                 (score descending, index ascending) against the scores staged in LDS, and the
//                 frame's kept rows in ascending order.
//   count_scan    exclusive scan of the per-frame kept counts.
//   token_gather  copies the kept rows into the compacted stream and writes their indices.
#include "sharpv_kernels.hpp"

namespace sharpv {

// ---------------------------------------------------------------------------- frame mean (Eq.2)
template <typename T>
__global__ __launch_bounds__(1024) void frame_mean_kernel(const T* __restrict__ feats, int f, int d,
                                                          float* __restrict__ mean) {
    __shared__ float sm[32][kBlockElems];
    const int t = blockIdx.x;
    const int slab = blockIdx.y;
    const int g = threadIdx.x >> 5;          // row class
    const int l = threadIdx.x & 31;          // chunk inside the slab
    const int c = slab * kBlockChunks + l;   // chunk inside the row
    const bool live = c < d / kChunk;
    float p[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) p[k] = 0.0f;
    if (live) {
        const T* col = feats + (size_t)t * f * d + (size_t)c * kChunk;
        for (int i = g; i < f; i += 32) {
            float v[8];
            unpack(load_raw<T>(col + (size_t)i * d), v);
#pragma unroll
            for (int k = 0; k < 8; ++k) p[k] = p[k] + v[k];
        }
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) sm[g][l * 8 + k] = p[k];
    for (int s = 16; s >= 1; s >>= 1) {
        __syncthreads();
        if (g < s) {
#pragma unroll
            for (int k = 0; k < 8; ++k) sm[g][l * 8 + k] = sm[g][l * 8 + k] + sm[g + s][l * 8 + k];
        }
    }
    if (g == 0 && live) {
        const float ff = (float)f;
        float* out = mean + (size_t)t * d + (size_t)c * kChunk;
#pragma unroll
        for (int k = 0; k < 8; ++k) out[k] = sm[0][l * 8 + k] / ff;
    }
}

// ---------------------------------------------------------------------------- per-token inner products
template <typename T>
__global__ __launch_bounds__(256) void token_dots_kernel(const T* __restrict__ feats, const float* __restrict__ mean,
                                                         int n_rows, int f, int d,
                                                         float* __restrict__ aa, float* __restrict__ am,
                                                         float* __restrict__ ab) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= n_rows) return;
    const int t = row / f;
    const bool has_prev = t > 0;
    const int nchunks = d / kChunk;
    const T* x = feats + (size_t)row * d;
    const T* xp = has_prev ? x - (size_t)f * d : x;
    const float* m = mean + (size_t)t * d;
    float s_aa = 0.0f, s_am = 0.0f, s_ab = 0.0f;
    for (int c0 = 0; c0 < nchunks; c0 += 64) {
        const int c = c0 + lane;
        float paa = 0.0f, pam = 0.0f, pab = 0.0f;
        if (c < nchunks) {
            const RawChunk<T> rx = load_raw<T>(x + (size_t)c * kChunk);
            const RawChunk<T> rp = load_raw<T>(xp + (size_t)c * kChunk);
            const RawChunk<float> rm = load_raw<float>(m + (size_t)c * kChunk);
            float a[8], b[8], mm[8];
            unpack(rx, a);
            unpack(rp, b);
            unpack(rm, mm);
            paa = chain8(a, a);
            pam = chain8(a, mm);
            pab = chain8(a, b);
        }
        paa = tree32(paa);
        pam = tree32(pam);
        pab = tree32(pab);
        const bool odd = c0 + kBlockChunks < nchunks;
        s_aa = add_blocks(s_aa, paa, odd);
        s_am = add_blocks(s_am, pam, odd);
        s_ab = add_blocks(s_ab, pab, odd);
    }
    if (lane == 0) {
        aa[row] = s_aa;
        am[row] = s_am;
        ab[row] = has_prev ? s_ab : 0.0f;
    }
}

// ---------------------------------------------------------------------------- scores, ratio, top-k
__global__ __launch_bounds__(1024) void frame_select_kernel(const float* __restrict__ mean, const float* __restrict__ aa,
                                                            const float* __restrict__ am, const float* __restrict__ ab,
                                                            const int32_t* __restrict__ frame_offsets, int B,
                                                            int f, int d, float w, int mode, float Kthr, int min_keep,
                                                            int32_t* __restrict__ local_idx,
                                                            int32_t* __restrict__ out_counts,
                                                            float* __restrict__ out_scores,
                                                            float* __restrict__ out_ratio) {
    __shared__ float sI[1024];
    __shared__ float sTT[1024];
    __shared__ float sblk[256];
    __shared__ float s_mm;
    __shared__ int s_first;
    __shared__ int s_k;
    __shared__ int wave_cnt[16];

    const int t = blockIdx.x;
    const int tid = threadIdx.x;
    const int nthreads = blockDim.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int nchunks = d / kChunk;
    const int nblocks = (nchunks + kBlockChunks - 1) / kBlockChunks;

    // mean.mean in the common order: one half-wavefront per 256-element block
    {
        const float* m = mean + (size_t)t * d;
        const int half = tid >> 5, hl = tid & 31, nhalves = nthreads >> 5;
        for (int b0 = 0; b0 < nblocks; b0 += nhalves) {
            const int b = b0 + half;
            const int c = b * kBlockChunks + hl;
            float v = 0.0f;
            if (b < nblocks && c < nchunks) {
                float x[8];
                unpack(load_raw<float>(m + (size_t)c * kChunk), x);
                v = chain8(x, x);
            }
            v = tree32(v);
            if (hl == 0 && b < nblocks) sblk[b] = v;
        }
    }
    if (tid == 0) s_first = (frame_offsets == nullptr) ? (t == 0) : 0;
    __syncthreads();
    if (frame_offsets != nullptr)
        for (int b = tid; b < B; b += nthreads)
            if (frame_offsets[b] == t) s_first = 1;          // first frame of a video (Eq.6)
    if (tid == 0) {
        float acc = 0.0f;
        for (int b = 0; b < nblocks; ++b) acc = acc + sblk[b];
        s_mm = acc;
    }
    __syncthreads();
    const float mm = s_mm;
    const bool first = s_first != 0 || t == 0;

    // Eq.1-4 per token
    const int i = tid;
    float score = 0.0f;
    if (i < f) {
        const size_t r = (size_t)t * f + i;
        const float xx = aa[r];
        const float S = dissim_from_dots(am[r], xx, mm);                     // Eq.2
        const float T = first ? S : dissim_from_dots(ab[r], xx, aa[r - f]);  // Eq.3 (Eq.6 on a first frame)
        score = __builtin_fmaf(w, S, T);                                     // Eq.4
        sI[i] = score;
        sTT[i] = T * T;
        if (out_scores != nullptr) out_scores[r] = score;
    }
    __syncthreads();

    // Eq.5 / Eq.6: ||T_t||_2 / (2 sqrt f), the squares summed as 32 interleaved partials + halving tree
    if (wave == 0) {
        float p = 0.0f;
        if (lane < 32)
            for (int j = lane; j < f; j += 32) p = p + sTT[j];
        p = tree32(p);
        if (lane == 0) {
            float rt = __builtin_sqrtf(p) / (2.0f * __builtin_sqrtf((float)f));
            rt = rt > 1.0f ? 1.0f : rt;
            rt = rt < 0.0f ? 0.0f : rt;
            const float prod = rt * (float)f;
            int k = (int)__builtin_floorf(prod + 0.5f);
            k = k < min_keep ? min_keep : k;
            k = k > f ? f : k;
            s_k = k;
            if (out_ratio != nullptr) out_ratio[t] = rt;
        }
    }
    __syncthreads();

    // top-k by counting: token i is kept iff fewer than k tokens are ahead of it
    // (higher score, or the same score and a lower index)
    int keep = 0;
    if (i < f) {
        if (mode == 0) {
            const int k = s_k;
            int rank = 0;
            for (int j = 0; j < f; ++j) {
                const float v = sI[j];
                rank += (v > score) || (v == score && j < i);
            }
            keep = rank < k;
        } else {
            keep = score >= Kthr;
        }
    }
    const unsigned long long bal = __ballot(keep != 0);
    const int before = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) wave_cnt[wave] = __popcll(bal);
    __syncthreads();
    int base = 0, total = 0;
    for (int q = 0; q < (nthreads >> 6); ++q) {
        const int cq = wave_cnt[q];
        base += q < wave ? cq : 0;
        total += cq;
    }
    if (keep) local_idx[(size_t)t * f + base + before] = t * f + i;
    if (tid == 0) out_counts[t] = total;
}

// ---------------------------------------------------------------------------- exclusive scan of the counts
__global__ __launch_bounds__(1024) void count_scan_kernel(const int32_t* __restrict__ counts, int n,
                                                          int32_t* __restrict__ offsets) {
    __shared__ int part[1024];
    const int tid = threadIdx.x;
    const int seg = (n + 1023) / 1024;
    const int lo = tid * seg;
    const int hi = lo + seg < n ? lo + seg : n;
    int s = 0;
    for (int j = lo; j < hi; ++j) s += counts[j];
    part[tid] = s;
    __syncthreads();
    for (int step = 1; step < 1024; step <<= 1) {
        const int v = tid >= step ? part[tid - step] : 0;
        __syncthreads();
        part[tid] += v;
        __syncthreads();
    }
    int run = part[tid] - s;                 // exclusive prefix of this thread's segment
    for (int j = lo; j < hi; ++j) {
        offsets[j] = run;
        run += counts[j];
    }
    if (tid == 1023) offsets[n] = part[1023];
}

// ---------------------------------------------------------------------------- compaction
constexpr int kGatherSplit = 4;     // workgroups per frame
__global__ __launch_bounds__(256) void token_gather_kernel(const char* __restrict__ feats, int f, int row_bytes,
                                                           const int32_t* __restrict__ local_idx,
                                                           const int32_t* __restrict__ counts,
                                                           const int32_t* __restrict__ offsets,
                                                           int32_t* __restrict__ out_idx, char* __restrict__ out_feats) {
    const int t = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int q = blockIdx.y * 4 + (threadIdx.x >> 6);
    const int cnt = counts[t];
    const int off = offsets[t];
    const int units = row_bytes / 16;
    for (int r = q; r < cnt; r += kGatherSplit * 4) {
        const int src_row = local_idx[(size_t)t * f + r];
        const uint4* src = reinterpret_cast<const uint4*>(feats + (size_t)src_row * row_bytes);
        uint4* dst = reinterpret_cast<uint4*>(out_feats + (size_t)(off + r) * row_bytes);
        for (int u = lane; u < units; u += 64) dst[u] = src[u];
        if (lane == 0) out_idx[off + r] = src_row;
    }
}

// ---------------------------------------------------------------------------- host side
int launch_prune_tokens(const TokArgs& a) {
    hipStream_t st = a.stream;
    TokWorkspace ws = carve_tok_workspace(a.workspace, a.n, a.f, a.d);
    const int n_rows = a.n * a.f;
    const int slabs = (a.d + kBlockElems - 1) / kBlockElems;
    const size_t esz = a.dtype == SHARPV_F32 ? 4 : 2;

    {
        TimedLaunch tl(kFrameMean, st);
        if (a.dtype == SHARPV_BF16)
            hipLaunchKernelGGL(frame_mean_kernel<bf16_t>, dim3(a.n, slabs), dim3(1024), 0, st,
                               (const bf16_t*)a.feats, a.f, a.d, ws.mean);
        else
            hipLaunchKernelGGL(frame_mean_kernel<float>, dim3(a.n, slabs), dim3(1024), 0, st,
                               (const float*)a.feats, a.f, a.d, ws.mean);
    }
    if (hipGetLastError() != hipSuccess) return SHARPV_ERR_DEVICE;

    {
        TimedLaunch tl(kTokenDots, st);
        if (a.dtype == SHARPV_BF16)
            hipLaunchKernelGGL(token_dots_kernel<bf16_t>, dim3((n_rows + 3) / 4), dim3(256), 0, st,
                               (const bf16_t*)a.feats, (const float*)ws.mean, n_rows, a.f, a.d, ws.aa, ws.am, ws.ab);
        else
            hipLaunchKernelGGL(token_dots_kernel<float>, dim3((n_rows + 3) / 4), dim3(256), 0, st,
                               (const float*)a.feats, (const float*)ws.mean, n_rows, a.f, a.d, ws.aa, ws.am, ws.ab);
    }
    if (hipGetLastError() != hipSuccess) return SHARPV_ERR_DEVICE;

    {
        TimedLaunch tl(kFrameSelect, st);
        const int threads = (a.f + 63) / 64 * 64;
        hipLaunchKernelGGL(frame_select_kernel, dim3(a.n), dim3(threads), 0, st, (const float*)ws.mean,
                           (const float*)ws.aa, (const float*)ws.am, (const float*)ws.ab, a.frame_offsets, a.B,
                           a.f, a.d, a.w, a.mode, a.K, a.min_keep, ws.local_idx, a.out_counts, a.out_scores,
                           a.out_ratio);
    }
    if (hipGetLastError() != hipSuccess) return SHARPV_ERR_DEVICE;

    {
        TimedLaunch tl(kCountScan, st);
        hipLaunchKernelGGL(count_scan_kernel, dim3(1), dim3(1024), 0, st, (const int32_t*)a.out_counts, a.n,
                           a.out_offsets);
    }
    if (hipGetLastError() != hipSuccess) return SHARPV_ERR_DEVICE;

    {
        TimedLaunch tl(kTokenGather, st);
        hipLaunchKernelGGL(token_gather_kernel, dim3(a.n, kGatherSplit), dim3(256), 0, st, (const char*)a.feats, a.f,
                           (int)(a.d * esz), (const int32_t*)ws.local_idx, (const int32_t*)a.out_counts,
                           (const int32_t*)a.out_offsets, a.out_idx, (char*)a.out_feats);
    }
    if (hipGetLastError() != hipSuccess) return SHARPV_ERR_DEVICE;
    return SHARPV_OK;
}

}  // namespace sharpv
