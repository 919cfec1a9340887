// Intra-LLM stage (Sec. 3.2, Eq.7): per-token cosine between layer hidden state and original
// embedding, keep/discard decision, and the gather of the layer's K/V rows into a compacted cache.
//
// Kernels
//   kv_cosine   one wavefront per packed position; 64 positions per workgroup.  Streams the hidden
//               row and the original row once (16-byte loads, 1 KB contiguous per wavefront and
//               instruction), accumulates h.h, o.o, h.o in the fixed order of sharpv_device.hpp,
//               decides Eq.7 and leaves a 64-bit keep mask and a kept count per workgroup.
//   kv_mean     one workgroup per sequence: mean cosine of its visual tokens in a fixed order
//               (only launched when the mean is asked for or decides, kv_mode 1).
//   kv_gather   one workgroup per 64 positions: output offset = sum of the kept counts of the
//               preceding groups, rank inside the group by popcount, then 16-byte copies of the
//               kept K and V rows of every head.  A last workgroup writes the per-sequence counts.
#include "sharpv_kernels.hpp"

namespace sharpv {

// Where packed position s sits: returns true and the row of `orig` when s is a visual token.
__device__ __forceinline__ bool locate_visual(const SeqDesc& sd, int s, int* orig_row, int* seq) {
    if (sd.seq_offsets == nullptr) {
        const int rel = s - sd.vis_start0;
        *orig_row = rel;
        *seq = 0;
        return rel >= 0 && rel < sd.n_vis;
    }
    int b = 0;
    while (b + 1 < sd.B && sd.seq_offsets[b + 1] <= s) ++b;
    const int rel = s - sd.seq_offsets[b] - sd.vis_start[b];
    const int lo = sd.vis_offsets[b];
    *orig_row = lo + rel;
    *seq = b;
    return rel >= 0 && rel < sd.vis_offsets[b + 1] - lo;
}

template <typename T>
__global__ __launch_bounds__(256) void kv_cosine_kernel(const T* __restrict__ hidden, const T* __restrict__ orig,
                                                        SeqDesc sd, int S, int d, float M,
                                                        float* __restrict__ cos_out,       // [n_vis] or nullptr
                                                        unsigned long long* __restrict__ group_mask,
                                                        int32_t* __restrict__ group_count) {
    __shared__ int keep_flag[kGroup];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int group = blockIdx.x;
    const int nchunks = d / kChunk;

    for (int j = 0; j < kGroup / 4; ++j) {
        const int slot = j * 4 + wave;
        const int s = group * kGroup + slot;
        int keep = 0;
        if (s < S) {
            keep = 1;                                   // system / instruction tokens are always kept
            int p, b;
            if (locate_visual(sd, s, &p, &b)) {
                const T* hrow = hidden + (size_t)s * d;
                const T* orow = orig + (size_t)p * d;
                float hh = 0.0f, oo = 0.0f, ho = 0.0f;
                for (int c0 = 0; c0 < nchunks; c0 += 64) {
                    const int c = c0 + lane;
                    float phh = 0.0f, poo = 0.0f, pho = 0.0f;
                    if (c < nchunks) {
                        const RawChunk<T> rh = load_raw<T>(hrow + (size_t)c * kChunk);
                        const RawChunk<T> ro = load_raw<T>(orow + (size_t)c * kChunk);
                        float h[8], o[8];
                        unpack(rh, h);
                        unpack(ro, o);
                        phh = chain8(h, h);
                        poo = chain8(o, o);
                        pho = chain8(h, o);
                    }
                    phh = tree32(phh);
                    poo = tree32(poo);
                    pho = tree32(pho);
                    const bool odd = c0 + kBlockChunks < nchunks;
                    hh = add_blocks(hh, phh, odd);
                    oo = add_blocks(oo, poo, odd);
                    ho = add_blocks(ho, pho, odd);
                }
                const float c = cos_from_dots(ho, hh, oo);
                keep = !(c < M);                        // Eq.7: discard iff cos < M
                if (lane == 0 && cos_out != nullptr) cos_out[p] = c;
            }
        }
        if (lane == 0) keep_flag[slot] = keep;
    }
    __syncthreads();
    if (wave == 0) {
        const unsigned long long m = __ballot(keep_flag[lane] != 0);
        if (lane == 0) {
            group_mask[group] = m;
            group_count[group] = __popcll(m);
        }
    }
}

// Mean cosine of each sequence's visual tokens: 32 interleaved partial sums (token i goes to partial
// i % 32, ascending), halving tree, divided by the token count.  In kv_mode 1 also the decision.
__global__ __launch_bounds__(64) void kv_mean_kernel(const float* __restrict__ cosv, SeqDesc sd, float M,
                                                     float* __restrict__ mean_out,     // [B] or nullptr
                                                     int32_t* __restrict__ drop_seq) { // [B]
    const int b = blockIdx.x;
    const int lane = threadIdx.x;
    int lo = 0, hi = sd.n_vis;
    if (sd.seq_offsets != nullptr) {
        lo = sd.vis_offsets[b];
        hi = sd.vis_offsets[b + 1];
    }
    float p = 0.0f;
    if (lane < 32)
        for (int i = lo + lane; i < hi; i += 32) p = p + cosv[i];
    p = tree32(p);
    const float mean = hi > lo ? p / (float)(hi - lo) : 0.0f;
    if (lane == 0) {
        if (mean_out != nullptr) mean_out[b] = mean;
        drop_seq[b] = (hi > lo && mean < M) ? 1 : 0;
    }
}

// kv_mode 1: rebuild the keep masks from the per-sequence decision.
__global__ __launch_bounds__(64) void kv_mask_from_mean_kernel(SeqDesc sd, int S, const int32_t* __restrict__ drop_seq,
                                                               unsigned long long* __restrict__ group_mask,
                                                               int32_t* __restrict__ group_count) {
    const int group = blockIdx.x;
    const int lane = threadIdx.x;
    const int s = group * kGroup + lane;
    int keep = 0;
    if (s < S) {
        int p, b;
        keep = locate_visual(sd, s, &p, &b) ? (drop_seq[b] == 0) : 1;
    }
    const unsigned long long m = __ballot(keep != 0);
    if (lane == 0) {
        group_mask[group] = m;
        group_count[group] = __popcll(m);
    }
}

__device__ __forceinline__ int block_sum_int(int v, int* scratch) {
    // integer sum over the workgroup (order is irrelevant for integers)
    for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) scratch[wave] = v;
    __syncthreads();
    int tot = 0;
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) tot += scratch[w];
    __syncthreads();
    return tot;
}

__device__ __forceinline__ int kept_before(const unsigned long long* group_mask, const int32_t* group_count,
                                           int pos, int* scratch) {
    // number of kept positions in [0, pos): whole groups by their counts, the rest by popcount
    const int g = pos / kGroup;
    int part = 0;
    for (int j = threadIdx.x; j < g; j += blockDim.x) part += group_count[j];
    int tot = block_sum_int(part, scratch);
    const int r = pos % kGroup;
    if (r) tot += __popcll(group_mask[g] & ((1ull << r) - 1ull));
    return tot;
}

__global__ __launch_bounds__(256) void kv_gather_kernel(const char* __restrict__ K, const char* __restrict__ V,
                                                        long long stride_h_bytes, long long stride_s_bytes,
                                                        char* __restrict__ K_out, char* __restrict__ V_out,
                                                        long long out_stride_h_bytes, int row_bytes, int H,
                                                        SeqDesc sd, int S, int n_groups,
                                                        const unsigned long long* __restrict__ group_mask,
                                                        const int32_t* __restrict__ group_count,
                                                        int32_t* __restrict__ out_idx, int32_t* __restrict__ out_count) {
    __shared__ int scratch[4];
    __shared__ int src_slot[kGroup];
    const int group = blockIdx.x;

    if (group == n_groups) {                     // extra workgroup: kept positions per sequence
        if (sd.seq_offsets == nullptr) {
            const int tot = kept_before(group_mask, group_count, S, scratch);
            if (threadIdx.x == 0) out_count[0] = tot;
        } else {
            for (int b = 0; b < sd.B; ++b) {
                const int lo = kept_before(group_mask, group_count, sd.seq_offsets[b], scratch);
                const int hi = kept_before(group_mask, group_count, sd.seq_offsets[b + 1], scratch);
                if (threadIdx.x == 0) out_count[b] = hi - lo;
            }
        }
        return;
    }

    const int base = kept_before(group_mask, group_count, group * kGroup, scratch);
    const unsigned long long mask = group_mask[group];
    const int cnt = __popcll(mask);
    if (threadIdx.x < kGroup) {
        const int l = threadIdx.x;
        if ((mask >> l) & 1ull) {
            const int r = __popcll(mask & ((1ull << l) - 1ull));
            src_slot[r] = l;
            out_idx[base + r] = group * kGroup + l;
        }
    }
    __syncthreads();
    if (K == nullptr) return;

    // copy units of 16 bytes: (kept row r, tensor K|V, head h, 16-byte piece q)
    const int pieces = row_bytes / 16;
    const int per_row = 2 * H * pieces;
    const int total = cnt * per_row;
    for (int u = threadIdx.x; u < total; u += blockDim.x) {
        const int r = u / per_row;
        int rem = u - r * per_row;
        const int kv = rem / (H * pieces);
        rem -= kv * H * pieces;
        const int h = rem / pieces;
        const int q = rem - h * pieces;
        const long long s = (long long)group * kGroup + src_slot[r];
        const char* src = (kv ? V : K) + h * stride_h_bytes + s * stride_s_bytes + (long long)q * 16;
        char* dst = (kv ? V_out : K_out) + h * out_stride_h_bytes + (long long)(base + r) * row_bytes + (long long)q * 16;
        *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
    }
}

// ---------------------------------------------------------------------------- host side
int launch_prune_kv(const KvArgs& a) {
    hipStream_t st = a.stream;
    const int n_groups = (a.S + kGroup - 1) / kGroup;
    KvWorkspace ws = carve_kv_workspace(a.workspace, a.B, a.S, a.n_vis);
    float* cos_buf = a.out_cos != nullptr ? a.out_cos : ws.cosv;
    const bool need_mean = a.kv_mode == 1 || a.out_mean_cos != nullptr;
    float* cos_dst = (need_mean || a.out_cos != nullptr) ? cos_buf : nullptr;
    const size_t esz = a.dtype == SHARPV_F32 ? 4 : 2;

    {
        TimedLaunch tl(kKvCosine, st);
        if (a.dtype == SHARPV_BF16)
            hipLaunchKernelGGL(kv_cosine_kernel<bf16_t>, dim3(n_groups), dim3(256), 0, st, (const bf16_t*)a.hidden,
                               (const bf16_t*)a.orig, a.sd, a.S, a.d, a.M, cos_dst, ws.group_mask, ws.group_count);
        else
            hipLaunchKernelGGL(kv_cosine_kernel<float>, dim3(n_groups), dim3(256), 0, st, (const float*)a.hidden,
                               (const float*)a.orig, a.sd, a.S, a.d, a.M, cos_dst, ws.group_mask, ws.group_count);
    }
    if (hipGetLastError() != hipSuccess) return SHARPV_ERR_DEVICE;

    if (need_mean) {
        {
            TimedLaunch tl(kKvMean, st);
            hipLaunchKernelGGL(kv_mean_kernel, dim3(a.B), dim3(64), 0, st, (const float*)cos_buf, a.sd, a.M,
                               a.out_mean_cos, ws.drop_seq);
        }
        if (hipGetLastError() != hipSuccess) return SHARPV_ERR_DEVICE;
        if (a.kv_mode == 1) {
            hipLaunchKernelGGL(kv_mask_from_mean_kernel, dim3(n_groups), dim3(64), 0, st, a.sd, a.S,
                               (const int32_t*)ws.drop_seq, ws.group_mask, ws.group_count);
            if (hipGetLastError() != hipSuccess) return SHARPV_ERR_DEVICE;
        }
    }

    {
        TimedLaunch tl(kKvGather, st);
        hipLaunchKernelGGL(kv_gather_kernel, dim3(n_groups + 1), dim3(256), 0, st, (const char*)a.K, (const char*)a.V,
                           (long long)(a.kv_stride_h * (int64_t)esz), (long long)(a.kv_stride_s * (int64_t)esz),
                           (char*)a.K_out, (char*)a.V_out, (long long)(a.out_stride_h * (int64_t)esz),
                           (int)(a.D * esz), a.H, a.sd, a.S, n_groups, (const unsigned long long*)ws.group_mask,
                           (const int32_t*)ws.group_count, a.out_idx, a.out_count);
    }
    if (hipGetLastError() != hipSuccess) return SHARPV_ERR_DEVICE;
    return SHARPV_OK;
}

}  // namespace sharpv
