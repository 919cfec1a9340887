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

// Three inner products of one (hidden row, original row) pair by one wavefront, chunk index
// c = 64*q + lane in sweep q, with all loads of the row issued before the arithmetic starts.
// NS = number of sweeps (d <= 512*NS); FULL = every lane of every sweep holds a chunk (d == 512*NS).
template <typename T, int NS, bool FULL>
__device__ __forceinline__ float row_cosine(const T* __restrict__ hrow, const T* __restrict__ orow,
                                            int nchunks, int lane) {
    RawChunk<T> rh[NS], ro[NS];
#pragma unroll
    for (int q = 0; q < NS; ++q) {
        const int c = q * 64 + lane;
        if (FULL || c < nchunks) {
            rh[q] = load_raw<T>(hrow + (size_t)c * kChunk);
            ro[q] = load_raw<T>(orow + (size_t)c * kChunk);
        } else {
            rh[q] = zero_raw<T>();
            ro[q] = zero_raw<T>();
        }
    }
    float hh = 0.0f, oo = 0.0f, ho = 0.0f;
#pragma unroll
    for (int q = 0; q < NS; ++q) {
        float h[8], o[8];
        unpack(rh[q], h);
        unpack(ro[q], o);
        const float pair = tree32_pair(chain8(h, h), chain8(o, o));   // rows 0,2: h.h   rows 1,3: o.o
        const float single = tree32(chain8(h, o));
        const bool odd = FULL || (q * 64 + kBlockChunks < nchunks);    // does the sweep's second block exist
        hh = hh + lane_value(pair, 0);
        oo = oo + lane_value(pair, 16);
        ho = ho + lane_value(single, 0);
        if (odd) {
            hh = hh + lane_value(pair, 32);
            oo = oo + lane_value(pair, 48);
            ho = ho + lane_value(single, 32);
        }
    }
    return cos_from_dots(ho, hh, oo);
}

// Any d: sweeps in a loop (used when d > 4096).
template <typename T>
__device__ __forceinline__ float row_cosine_loop(const T* __restrict__ hrow, const T* __restrict__ orow,
                                                 int nchunks, int lane) {
    float hh = 0.0f, oo = 0.0f, ho = 0.0f;
    for (int c0 = 0; c0 < nchunks; c0 += 64) {
        const int c = c0 + lane;
        float phh = 0.0f, poo = 0.0f, pho = 0.0f;
        if (c < nchunks) {
            float h[8], o[8];
            unpack(load_raw<T>(hrow + (size_t)c * kChunk), h);
            unpack(load_raw<T>(orow + (size_t)c * kChunk), o);
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
    return cos_from_dots(ho, hh, oo);
}

constexpr int kCosWaves = 4;        // wavefronts per workgroup of kv_cosine

template <typename T, int NS, bool FULL>
__global__ __launch_bounds__(kCosWaves * 64) void kv_cosine_kernel(const T* __restrict__ hidden,
                                                                   const T* __restrict__ orig, SeqDesc sd, int S, int d,
                                                                   float M, float* __restrict__ cos_out,   // [n_vis] or nullptr
                                                                   unsigned long long* __restrict__ group_mask,
                                                                   int32_t* __restrict__ group_count) {
    __shared__ int keep_flag[kGroup];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int group = blockIdx.x;
    const int nchunks = d / kChunk;

    for (int j = 0; j < kGroup / kCosWaves; ++j) {
        const int slot = j * kCosWaves + wave;
        const int s = group * kGroup + slot;
        int keep = 0;
        if (s < S) {
            keep = 1;                                   // system / instruction tokens are always kept
            int p, b;
            if (locate_visual(sd, s, &p, &b)) {
                const T* hrow = hidden + (size_t)s * d;
                const T* orow = orig + (size_t)p * d;
                float c;
                if constexpr (NS > 0) c = row_cosine<T, NS, FULL>(hrow, orow, nchunks, lane);
                else c = row_cosine_loop<T>(hrow, orow, nchunks, lane);
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

template <typename T>
static void launch_kv_cosine(const KvArgs& a, const KvWorkspace& ws, float* cos_dst, int n_groups) {
    const int nchunks = a.d / kChunk;
    const int ns = (nchunks + 63) / 64;
    const bool full = nchunks == ns * 64;
    const dim3 grid(n_groups), block(kCosWaves * 64);
#define SHARPV_COS_CASE(NS_)                                                                                        \
    case NS_:                                                                                                       \
        if (full)                                                                                                   \
            hipLaunchKernelGGL((kv_cosine_kernel<T, NS_, true>), grid, block, 0, a.stream, (const T*)a.hidden,      \
                               (const T*)a.orig, a.sd, a.S, a.d, a.M, cos_dst, ws.group_mask, ws.group_count);     \
        else                                                                                                        \
            hipLaunchKernelGGL((kv_cosine_kernel<T, NS_, false>), grid, block, 0, a.stream, (const T*)a.hidden,     \
                               (const T*)a.orig, a.sd, a.S, a.d, a.M, cos_dst, ws.group_mask, ws.group_count);     \
        break;
    switch (ns) {
        SHARPV_COS_CASE(1) SHARPV_COS_CASE(2) SHARPV_COS_CASE(3) SHARPV_COS_CASE(4)
        SHARPV_COS_CASE(5) SHARPV_COS_CASE(6) SHARPV_COS_CASE(7) SHARPV_COS_CASE(8)
        default:
            hipLaunchKernelGGL((kv_cosine_kernel<T, 0, false>), grid, block, 0, a.stream, (const T*)a.hidden,
                               (const T*)a.orig, a.sd, a.S, a.d, a.M, cos_dst, ws.group_mask, ws.group_count);
    }
#undef SHARPV_COS_CASE
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

    // Copy in units of 16 bytes.  One kept position owns per_pos = 2*H*pieces units (K then V, head
    // by head); a wavefront takes one kept position at a time, lane -> unit, so the source position
    // is uniform and the per-lane offsets are computed once, outside the loop.
    const int pieces = row_bytes / 16;
    const int per_pos = 2 * H * pieces;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int nwaves = blockDim.x >> 6;
    for (int v0 = 0; v0 < per_pos; v0 += 64) {
        const int v = v0 + lane;
        const bool live = v < per_pos;
        const int kv = live ? v / (H * pieces) : 0;
        const int rem = live ? v - kv * H * pieces : 0;
        const int h = rem / pieces;
        const int q = rem - h * pieces;
        const char* src0 = (kv ? V : K) + h * stride_h_bytes + (long long)q * 16;
        char* dst0 = (kv ? V_out : K_out) + h * out_stride_h_bytes + (long long)q * 16;
        int r = wave;
        for (; r + 3 * nwaves < cnt; r += 4 * nwaves) {           // four positions in flight per wavefront
            uint4 t[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const long long s = (long long)group * kGroup + src_slot[r + k * nwaves];
                if (live) t[k] = *reinterpret_cast<const uint4*>(src0 + s * stride_s_bytes);
            }
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (live) *reinterpret_cast<uint4*>(dst0 + (long long)(base + r + k * nwaves) * row_bytes) = t[k];
        }
        for (; r < cnt; r += nwaves) {
            const long long s = (long long)group * kGroup + src_slot[r];
            if (live)
                *reinterpret_cast<uint4*>(dst0 + (long long)(base + r) * row_bytes) =
                    *reinterpret_cast<const uint4*>(src0 + s * stride_s_bytes);
        }
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
        if (a.dtype == SHARPV_BF16) launch_kv_cosine<bf16_t>(a, ws, cos_dst, n_groups);
        else launch_kv_cosine<float>(a, ws, cos_dst, n_groups);
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
