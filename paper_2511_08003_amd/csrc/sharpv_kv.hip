// Intra-LLM stage (Sec. 3.2, Eq.7): per-token cosine between layer hidden state and original
// embedding, keep/discard decision, and the gather of the layer's K/V rows into a compacted cache.
//
// Kernels
//   kv_cosine   one wavefront per packed position, 16 positions per workgroup.  A wavefront issues
//               all 16-byte loads of its hidden row and original row at once (1 KB contiguous per
//               instruction), accumulates h.h, o.o, h.o in the fixed order of sharpv_device.hpp and
//               decides Eq.7; the workgroup leaves one 16-bit word of the keep mask.
//   kv_mean     one workgroup per sequence: mean cosine of its visual tokens in a fixed order
//               (only launched when the mean is asked for or decides, kv_mode 1).
//   kv_gather   one workgroup per mask word (16 positions): output offset = popcount of the preceding
//               mask words, rank inside the word by popcount, then batched 16-byte copies of the kept
//               K and V rows, plane by plane.  A last workgroup writes the per-sequence counts.
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
            rh[q] = load_raw_stream<T>(hrow + (size_t)c * kChunk);
            ro[q] = load_raw_stream<T>(orow + (size_t)c * kChunk);
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

constexpr int kCosRows = kMaskWord;  // packed positions (= wavefronts) per workgroup of kv_cosine

// One wavefront per packed position, 16 positions per workgroup.  The 16 decisions of a workgroup
// form one 16-bit word of the keep mask; four consecutive words are the 64-bit mask of a group of
// kGroup = 64 positions (little endian: position 64g+i is bit i of 64-bit word g).
template <typename T, int NS, bool FULL>
__global__ __launch_bounds__(kCosRows * 64) void kv_cosine_kernel(const T* __restrict__ hidden,
                                                                  const T* __restrict__ orig, SeqDesc sd, int S, int d,
                                                                  float M, float* __restrict__ cos_out,   // [n_vis] or nullptr
                                                                  uint16_t* __restrict__ mask16) {
    __shared__ int keep_flag[kCosRows];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int s = blockIdx.x * kCosRows + wave;
    const int nchunks = d / kChunk;
    int keep = 0;
    if (s < S) {
        keep = 1;                                       // system / instruction tokens are always kept
        int p, b;
        if (locate_visual(sd, s, &p, &b)) {
            const T* hrow = hidden + (size_t)s * d;
            const T* orow = orig + (size_t)p * d;
            float c;
            if constexpr (NS > 0) c = row_cosine<T, NS, FULL>(hrow, orow, nchunks, lane);
            else c = row_cosine_loop<T>(hrow, orow, nchunks, lane);
            keep = !(c < M);                            // Eq.7: discard iff cos < M
            if (lane == 0 && cos_out != nullptr) cos_out[p] = c;
        }
    }
    if (lane == 0) keep_flag[wave] = keep;
    __syncthreads();
    if (wave == 0) {
        const unsigned long long m = __ballot(lane < kCosRows && keep_flag[lane & (kCosRows - 1)] != 0);
        if (lane == 0) mask16[blockIdx.x] = (uint16_t)m;
    }
}

template <typename T>
static void launch_kv_cosine(const KvArgs& a, const KvWorkspace& ws, float* cos_dst) {
    const int nchunks = a.d / kChunk;
    const int ns = (nchunks + 63) / 64;
    const bool full = nchunks == ns * 64;
    const dim3 grid((a.S + kCosRows - 1) / kCosRows), block(kCosRows * 64);
    uint16_t* mask16 = reinterpret_cast<uint16_t*>(ws.group_mask);
#define SHARPV_COS_CASE(NS_)                                                                                        \
    case NS_:                                                                                                       \
        if (full)                                                                                                   \
            hipLaunchKernelGGL((kv_cosine_kernel<T, NS_, true>), grid, block, 0, a.stream, (const T*)a.hidden,      \
                               (const T*)a.orig, a.sd, a.S, a.d, a.M, cos_dst, mask16);                             \
        else                                                                                                        \
            hipLaunchKernelGGL((kv_cosine_kernel<T, NS_, false>), grid, block, 0, a.stream, (const T*)a.hidden,     \
                               (const T*)a.orig, a.sd, a.S, a.d, a.M, cos_dst, mask16);                             \
        break;
    switch (ns) {
        SHARPV_COS_CASE(1) SHARPV_COS_CASE(2) SHARPV_COS_CASE(3) SHARPV_COS_CASE(4)
        SHARPV_COS_CASE(5) SHARPV_COS_CASE(6) SHARPV_COS_CASE(7) SHARPV_COS_CASE(8)
        default:
            hipLaunchKernelGGL((kv_cosine_kernel<T, 0, false>), grid, block, 0, a.stream, (const T*)a.hidden,
                               (const T*)a.orig, a.sd, a.S, a.d, a.M, cos_dst, mask16);
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
                                                               unsigned long long* __restrict__ group_mask) {
    const int group = blockIdx.x;
    const int lane = threadIdx.x;
    const int s = group * kGroup + lane;
    int keep = 0;
    if (s < S) {
        int p, b;
        keep = locate_visual(sd, s, &p, &b) ? (drop_seq[b] == 0) : 1;
    }
    const unsigned long long m = __ballot(keep != 0);
    if (lane == 0) group_mask[group] = m;
}

constexpr int kGatherThreads = 256;

// Number of kept positions in [0, pos), pos <= S, summed by the whole workgroup from the 16-bit mask
// words (every word below ceil(S/16) is complete: kv_cosine clears the bits of positions >= S).
__device__ __forceinline__ int kept_before(const uint16_t* __restrict__ mask16, int pos, int* scratch) {
    const int w16 = pos / kMaskWord;             // complete 16-bit words below pos
    const int w64 = w16 / 4;
    const unsigned long long* m64 = reinterpret_cast<const unsigned long long*>(mask16);
    int part = 0;
    for (int j = threadIdx.x; j < w64; j += kGatherThreads) part += __popcll(m64[j]);
    if ((int)threadIdx.x < w16 - w64 * 4) part += __popc((unsigned)mask16[w64 * 4 + threadIdx.x]);
    if (threadIdx.x == 0) {
        const int r = pos % kMaskWord;
        if (r) part += __popc((unsigned)mask16[w16] & ((1u << r) - 1u));
    }
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) part += __shfl_xor(part, s);
    __syncthreads();                             // scratch may still be read from a previous call
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = part;
    __syncthreads();
    int tot = 0;
#pragma unroll
    for (int w = 0; w < kGatherThreads / 64; ++w) tot += scratch[w];
    return tot;
}
constexpr int kGatherBatch = 8;     // 16-byte loads in flight per lane

// One workgroup per mask word (16 packed positions).  Its output offset is the number of kept positions
// before the word (popcounts of the preceding mask words, summed by the workgroup).  Kept row r of the
// word goes to output row offset + r of every K / V head plane; lanes walk (r, 16-byte piece) so that one wavefront reads
// and writes whole consecutive rows of one plane, and the planes are taken in batches with all loads
// of a batch issued before its stores.  CH = number of heads when known at compile time (the loads
// of a batch then carry no predicate, which is what lets them overlap); CH = 0 takes any H and
// clamps the plane index of the loads instead of predicating them.
template <int CH>
__global__ __launch_bounds__(kGatherThreads) void kv_gather_kernel(
    const char* __restrict__ K, const char* __restrict__ V, long long stride_h_bytes, long long stride_s_bytes,
    char* __restrict__ K_out, char* __restrict__ V_out, long long out_stride_h_bytes, int row_bytes, int H_any,
    const uint16_t* __restrict__ mask16, int n_words, SeqDesc sd, int S, int32_t* __restrict__ out_idx,
    int32_t* __restrict__ out_count) {
    __shared__ int scratch[kGatherThreads / 64];
    const int H = CH > 0 ? CH : H_any;
    const int word = blockIdx.x;
    if (word == n_words) {                       // extra workgroup: kept positions per sequence
        if (sd.seq_offsets == nullptr) {
            const int tot = kept_before(mask16, S, scratch);
            if (threadIdx.x == 0) out_count[0] = tot;
        } else {
            for (int b = 0; b < sd.B; ++b) {
                const int lo = kept_before(mask16, sd.seq_offsets[b], scratch);
                const int hi = kept_before(mask16, sd.seq_offsets[b + 1], scratch);
                if (threadIdx.x == 0) out_count[b] = hi - lo;
            }
        }
        return;
    }
    const unsigned mask = mask16[word];
    if (mask == 0u) return;                      // nothing kept here (uniform over the workgroup)
    const int base = kept_before(mask16, word * kMaskWord, scratch);
    const int cnt = __popc(mask);
    const int pieces = row_bytes / 16;
    const int units = cnt * pieces;              // 16-byte units of one plane of this word
    const int planes = 2 * H;                    // K heads, then V heads
    constexpr int kBatch = CH > 0 ? (2 * CH < kGatherBatch ? 2 * CH : kGatherBatch) : kGatherBatch;
    for (int w = threadIdx.x; w < units; w += kGatherThreads) {
        const int r = w / pieces;
        const int q = w - r * pieces;
        unsigned m = mask;                       // position of the r-th kept bit
        for (int i = 0; i < r; ++i) m &= m - 1u;
        const int pos = word * kMaskWord + (__ffs(m) - 1);
        if (q == 0) out_idx[base + r] = pos;
        if (K == nullptr) continue;
        const long long src_off = (long long)pos * stride_s_bytes + (long long)q * 16;
        const long long dst_off = (long long)(base + r) * row_bytes + (long long)q * 16;
        for (int p0 = 0; p0 < planes; p0 += kBatch) {
            uint4 t[kBatch];
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {
                int p = p0 + k;
                if (CH == 0) p = p < planes ? p : planes - 1;          // a valid plane, loaded twice
                const int h = p < H ? p : p - H;
                t[k] = load_stream(reinterpret_cast<const uint4*>((p < H ? K : V) + h * stride_h_bytes + src_off));
            }
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {
                const int p = p0 + k;
                if (CH > 0 || p < planes) {
                    const int h = p < H ? p : p - H;
                    store_stream(reinterpret_cast<uint4*>((p < H ? K_out : V_out) + h * out_stride_h_bytes + dst_off), t[k]);
                }
            }
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
        if (a.dtype == SHARPV_BF16) launch_kv_cosine<bf16_t>(a, ws, cos_dst);
        else launch_kv_cosine<float>(a, ws, cos_dst);
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
                               (const int32_t*)ws.drop_seq, ws.group_mask);
            if (hipGetLastError() != hipSuccess) return SHARPV_ERR_DEVICE;
        }
    }

    const int n_words = (a.S + kMaskWord - 1) / kMaskWord;
    const uint16_t* mask16 = reinterpret_cast<const uint16_t*>(ws.group_mask);
    {
        TimedLaunch tl(kKvGather, st);
#define SHARPV_GATHER(CH_)                                                                                          \
    hipLaunchKernelGGL((kv_gather_kernel<CH_>), dim3(n_words + 1), dim3(kGatherThreads), 0, st, (const char*)a.K,   \
                       (const char*)a.V, (long long)(a.kv_stride_h * (int64_t)esz),                                  \
                       (long long)(a.kv_stride_s * (int64_t)esz), (char*)a.K_out, (char*)a.V_out,                    \
                       (long long)(a.out_stride_h * (int64_t)esz), (int)(a.D * esz), a.H, mask16, n_words, a.sd,     \
                       a.S, a.out_idx, a.out_count)
        switch (a.H) {
            case 1: SHARPV_GATHER(1); break;
            case 2: SHARPV_GATHER(2); break;
            case 4: SHARPV_GATHER(4); break;
            case 8: SHARPV_GATHER(8); break;
            default: SHARPV_GATHER(0);
        }
#undef SHARPV_GATHER
    }
    if (hipGetLastError() != hipSuccess) return SHARPV_ERR_DEVICE;
    return SHARPV_OK;
}

}  // namespace sharpv
