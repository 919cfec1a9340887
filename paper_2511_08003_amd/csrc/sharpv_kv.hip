// Intra-LLM stage (Sec. 3.2, Eq.7): per-token cosine between layer hidden state and original
// embedding, keep/discard decision, and the gather of the layer's K/V rows into a compacted cache.
//
// Kernels
//   kv_cosine   one wavefront per packed position, 8 positions per workgroup.  A wavefront issues
//               all 16-byte loads of its hidden row and original row at once (1 KB contiguous per
//               instruction), accumulates h.h, o.o, h.o in the fixed order of sharpv_device.hpp and
//               decides Eq.7; the workgroup leaves one byte of the keep mask.
//   kv_mean     one workgroup per sequence: mean cosine of its visual tokens in a fixed order
//               (only launched when the mean is asked for or decides, kv_mode 1).
//   kv_gather   one workgroup per mask word (16 positions): output offset = popcount of the preceding
//               mask words, rank inside the word by popcount, then batched 16-byte copies of the kept
//               K and V rows, plane by plane.  One more workgroup per sequence writes that sequence's count.
//   kv_gather_rope  the same gather with the rotary position of every kept K row re-encoded for its
//               new place in the compacted cache (Sec. 4.1, Implementation Details).
#include "sharpv_kernels.hpp"

namespace sharpv {

// Sequence that owns packed position s (0 <= s < seq_offsets[B]): the last b with seq_offsets[b] <= s.
__device__ __forceinline__ int find_sequence(const SeqDesc& sd, int s) {
    int lo = 0, hi = sd.B;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (sd.seq_offsets[mid] <= s) lo = mid; else hi = mid;
    }
    return lo;
}

// Where packed position s sits: returns true and the row of `orig` when s is a visual token.
__device__ __forceinline__ bool locate_visual(const SeqDesc& sd, int s, int* orig_row, int* seq) {
    if (sd.orig_row != nullptr) {                // explicit map (sequence already thinned out by earlier layers)
        const int p = sd.orig_row[s];
        *orig_row = p;
        *seq = 0;
        return p >= 0 && p < sd.n_vis;
    }
    if (sd.seq_offsets == nullptr) {
        const int rel = s - sd.vis_start0;
        *orig_row = rel;
        *seq = 0;
        return rel >= 0 && rel < sd.n_vis;
    }
    const int b = find_sequence(sd, s);
    const int rel = s - sd.seq_offsets[b] - sd.vis_start[b];
    const int lo = sd.vis_offsets[b];
    const int p = lo + rel;
    *orig_row = p;
    *seq = b;
    // the last two tests only matter for malformed descriptor arrays: no row outside orig is ever read
    return rel >= 0 && rel < sd.vis_offsets[b + 1] - lo && p >= 0 && p < sd.n_vis;
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

constexpr int kCosRows = 8;          // packed positions (= wavefronts) per workgroup of kv_cosine: one byte of the mask

// One wavefront per packed position, 8 positions per workgroup (smaller workgroups keep more
// wavefronts resident while others retire).  The 8 decisions of a workgroup form one byte of the keep
// mask; two bytes are one 16-bit word, four words the 64-bit mask of a group of kGroup = 64 positions
// (little endian: position 64g+i is bit i of 64-bit word g).
template <typename T, int NS, bool FULL>
__global__ __launch_bounds__(kCosRows * 64) void kv_cosine_kernel(const T* __restrict__ hidden,
                                                                  const T* __restrict__ orig, SeqDesc sd, int S, int d,
                                                                  float M, float* __restrict__ cos_out,   // [n_vis] or nullptr
                                                                  uint8_t* __restrict__ mask8) {
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
            // by visual token, or by position when the visual tokens are given by a map
            if (lane == 0 && cos_out != nullptr) cos_out[sd.orig_row != nullptr ? s : p] = c;
        }
    }
    if (lane == 0) keep_flag[wave] = keep;
    __syncthreads();
    if (wave == 0) {
        const unsigned long long m = __ballot(lane < kCosRows && keep_flag[lane & (kCosRows - 1)] != 0);
        if (lane == 0) mask8[blockIdx.x] = (uint8_t)m;
    }
}

template <typename T>
static void launch_kv_cosine(const KvArgs& a, const KvWorkspace& ws, float* cos_dst) {
    const int nchunks = a.d / kChunk;
    const int ns = (nchunks + 63) / 64;
    const bool full = nchunks == ns * 64;
    // both bytes of every 16-bit mask word are written (the second one may lie wholly past S: zero)
    const dim3 grid(2 * ((a.S + kMaskWord - 1) / kMaskWord)), block(kCosRows * 64);
    uint8_t* mask16 = reinterpret_cast<uint8_t*>(ws.group_mask);
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
    if (sd.seq_offsets != nullptr) {             // clamped: malformed offsets must not reach past the cosines
        lo = min(max(sd.vis_offsets[b], 0), sd.n_vis);
        hi = min(max(sd.vis_offsets[b + 1], 0), sd.n_vis);
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

// Exclusive prefix of the kept positions over the 16-bit mask words (one workgroup; used for long
// sequences, where every gather workgroup adding up all the words before its own would be quadratic).
__global__ __launch_bounds__(1024) void kv_mask_scan_kernel(const uint16_t* __restrict__ mask16, int n_words,
                                                            int32_t* __restrict__ word_base) {
    __shared__ int wave_tot[16];
    const int tid = threadIdx.x;
    const int seg = (n_words + 1023) / 1024;
    const int lo = tid * seg < n_words ? tid * seg : n_words;
    const int hi = lo + seg < n_words ? lo + seg : n_words;
    int sum = 0;
    for (int j = lo; j < hi; ++j) sum += __popc((unsigned)mask16[j]);
    const int incl = block_inclusive_scan_1024(sum, wave_tot);
    int run = incl - sum;
    for (int j = lo; j < hi; ++j) {
        word_base[j] = run;
        run += __popc((unsigned)mask16[j]);
    }
    if (tid == 1023) word_base[n_words] = incl;
}

constexpr int kGatherThreads = 256;

// Number of kept positions in [0, pos), pos <= S: read from the scanned prefix when there is one, else
// summed by the whole workgroup from the 16-bit mask words (every word below ceil(S/16) is complete:
// kv_cosine clears the bits of positions >= S).  Called by all threads of the workgroup.
__device__ __forceinline__ int kept_before(const uint16_t* __restrict__ mask16,
                                           const int32_t* __restrict__ word_base, int pos, int* scratch) {
    if (word_base != nullptr) {                  // the prefix over the words is already there
        const int w = pos / kMaskWord, r = pos % kMaskWord;
        return word_base[w] + (r ? __popc((unsigned)mask16[w] & ((1u << r) - 1u)) : 0);
    }
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
// clamps the plane index of the loads instead of predicating them.  Workgroups n_words .. n_words+B-1
// write the kept count of one sequence each.
template <int CH>
__global__ __launch_bounds__(kGatherThreads) void kv_gather_kernel(
    const char* __restrict__ K, const char* __restrict__ V, long long stride_h_bytes, long long stride_s_bytes,
    char* __restrict__ K_out, char* __restrict__ V_out, long long out_stride_h_bytes, int row_bytes, int H_any,
    const uint16_t* __restrict__ mask16, const int32_t* __restrict__ word_base, int n_words, SeqDesc sd, int S,
    int32_t* __restrict__ out_idx, int32_t* __restrict__ out_count, int32_t* __restrict__ out_orig_row) {
    __shared__ int scratch[kGatherThreads / 64];
    const int H = CH > 0 ? CH : H_any;
    const int word = blockIdx.x;
    // With the number of heads unknown at compile time the grid's second dimension splits the head
    // planes, one batch per workgroup (many heads would otherwise be walked by too few threads).
    const bool first_slice = blockIdx.y == 0;
    if (word >= n_words) {                       // B extra workgroups: kept positions of one sequence each
        if (!first_slice) return;
        const int b = word - n_words;
        int p_lo = 0, p_hi = S;
        if (sd.seq_offsets != nullptr) {             // clamped: malformed offsets must not reach past the mask
            p_lo = min(max(sd.seq_offsets[b], 0), S);
            p_hi = min(max(sd.seq_offsets[b + 1], 0), S);
        }
        const int lo = kept_before(mask16, word_base, p_lo, scratch);
        const int hi = kept_before(mask16, word_base, p_hi, scratch);
        if (threadIdx.x == 0) out_count[b] = hi - lo;
        return;
    }
    const unsigned mask = mask16[word];
    if (mask == 0u) return;                      // nothing kept here (uniform over the workgroup)
    const int base = kept_before(mask16, word_base, word * kMaskWord, scratch);
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
        if (q == 0 && first_slice) {
            out_idx[base + r] = pos;
            if (out_orig_row != nullptr) {       // the next layer's map: the row behind each kept position
                const int p = sd.orig_row[pos];
                out_orig_row[base + r] = (p >= 0 && p < sd.n_vis) ? p : -1;
            }
        }
        if (K == nullptr) continue;
        const long long src_off = (long long)pos * stride_s_bytes + (long long)q * 16;
        const long long dst_off = (long long)(base + r) * row_bytes + (long long)q * 16;
        const int p_begin = CH > 0 ? 0 : (int)blockIdx.y * kBatch;
        const int p_end = CH > 0 ? planes : (p_begin + kBatch < planes ? p_begin + kBatch : planes);
        for (int p0 = p_begin; p0 < p_end; p0 += kBatch) {
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

// ---------------------------------------------------------------------------- gather with rotary re-encoding
// 16-byte piece <-> floats.  bf16 -> float32 is exact; float32 -> bf16 rounds to nearest, ties to even
// (finite values).
template <typename T> struct Piece;
template <> struct Piece<bf16_t> {
    static constexpr int kElems = 8;
    static __device__ __forceinline__ void widen(const uint4& q, float (&v)[8]) {
        v[0] = __uint_as_float(q.x << 16); v[1] = __uint_as_float(q.x & 0xffff0000u);
        v[2] = __uint_as_float(q.y << 16); v[3] = __uint_as_float(q.y & 0xffff0000u);
        v[4] = __uint_as_float(q.z << 16); v[5] = __uint_as_float(q.z & 0xffff0000u);
        v[6] = __uint_as_float(q.w << 16); v[7] = __uint_as_float(q.w & 0xffff0000u);
    }
    static __device__ __forceinline__ uint32_t round1(float f) {
        const uint32_t u = __float_as_uint(f);
        return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    }
    static __device__ __forceinline__ uint4 narrow(const float (&v)[8]) {
        return make_uint4(round1(v[0]) | (round1(v[1]) << 16), round1(v[2]) | (round1(v[3]) << 16),
                          round1(v[4]) | (round1(v[5]) << 16), round1(v[6]) | (round1(v[7]) << 16));
    }
};
template <> struct Piece<float> {
    static constexpr int kElems = 4;
    static __device__ __forceinline__ void widen(const uint4& q, float (&v)[4]) {
        v[0] = __uint_as_float(q.x); v[1] = __uint_as_float(q.y); v[2] = __uint_as_float(q.z); v[3] = __uint_as_float(q.w);
    }
    static __device__ __forceinline__ uint4 narrow(const float (&v)[4]) {
        return make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3]));
    }
};

// Pair (x, y) turned back by the angle whose cosine / sine are c / s (Sec. 4.1, Implementation Details:
// the positional embedding is re-encoded for the row's new place); the two products are rounded on
// their own, then one fused multiply-add each.
__device__ __forceinline__ void rotate_back(float x, float y, float c, float s, float* xn, float* yn) {
    const float ys = y * s;
    const float xs = x * s;
    *xn = __builtin_fmaf(x, c, ys);
    *yn = __builtin_fmaf(y, c, -xs);
}

// kv_gather with the rotary embedding of every kept K row re-encoded on the way: a row that sat at
// position p of its sequence and becomes that sequence's j-th kept row is turned back by delta = p - j
// steps, with cos / sin of delta * theta_i read from the caller's tables [rope_len][D/2].
// LAYOUT 0 pairs element i with i + D/2, LAYOUT 1 pairs 2i with 2i+1.  A thread owns the 16-byte pieces
// q and q + pieces/2 of a kept row (for LAYOUT 0 they hold the two halves of the same pairs) in every
// head plane; V rows are copied unchanged.  Everything else (output offset from the popcounts of the
// preceding mask words, rank inside the word, batched loads, extra workgroup for the counts) is as in
// kv_gather_kernel.
template <typename T, int LAYOUT, int CH>
__global__ __launch_bounds__(kGatherThreads) void kv_gather_rope_kernel(
    const char* __restrict__ K, const char* __restrict__ V, long long stride_h_bytes, long long stride_s_bytes,
    char* __restrict__ K_out, char* __restrict__ V_out, long long out_stride_h_bytes, int row_bytes, int H_any,
    const uint16_t* __restrict__ mask16, const int32_t* __restrict__ word_base, int n_words, SeqDesc sd, int S,
    int32_t* __restrict__ out_idx, int32_t* __restrict__ out_count, int32_t* __restrict__ out_orig_row,
    const float* __restrict__ rope_cos, const float* __restrict__ rope_sin, int rope_len) {
    __shared__ int scratch[kGatherThreads / 64];
    constexpr int E = Piece<T>::kElems;
    const int H = CH > 0 ? CH : H_any;
    const int word = blockIdx.x;
    const bool first_slice = blockIdx.y == 0;    // the grid's second dimension splits the heads when CH == 0
    if (word >= n_words) {                       // B extra workgroups: kept positions of one sequence each
        if (!first_slice) return;
        const int b = word - n_words;
        int p_lo = 0, p_hi = S;
        if (sd.seq_offsets != nullptr) {             // clamped: malformed offsets must not reach past the mask
            p_lo = min(max(sd.seq_offsets[b], 0), S);
            p_hi = min(max(sd.seq_offsets[b + 1], 0), S);
        }
        const int lo = kept_before(mask16, word_base, p_lo, scratch);
        const int hi = kept_before(mask16, word_base, p_hi, scratch);
        if (threadIdx.x == 0) out_count[b] = hi - lo;
        return;
    }
    const unsigned mask = mask16[word];
    if (mask == 0u) return;                      // nothing kept here (uniform over the workgroup)
    const int word_pos = word * kMaskWord;
    const int base = kept_before(mask16, word_base, word_pos, scratch);
    // sequence of the word's first position, and how many rows were kept before that sequence starts
    int b_first = 0, first_lo = 0, first_kept = 0;
    if (sd.seq_offsets != nullptr) {
        b_first = find_sequence(sd, word_pos);
        first_lo = min(max(sd.seq_offsets[b_first], 0), word_pos);     // clamped against malformed offsets
        first_kept = kept_before(mask16, word_base, first_lo, scratch);
    }
    const int cnt = __popc(mask);
    const int pieces = row_bytes / 16;
    const int hp = pieces / 2;                   // pieces per half row
    const int half = hp * E;                     // pairs per row = D / 2
    const int units = cnt * hp;
    for (int w = threadIdx.x; w < units; w += kGatherThreads) {
        const int r = w / hp;
        const int q = w - r * hp;
        unsigned m = mask;                       // position of the r-th kept bit
        for (int i = 0; i < r; ++i) m &= m - 1u;
        const int bit = __ffs(m) - 1;
        const int pos = word_pos + bit;
        if (q == 0 && first_slice) {
            out_idx[base + r] = pos;
            if (out_orig_row != nullptr) {       // the next layer's map: the row behind each kept position
                const int p = sd.orig_row[pos];
                out_orig_row[base + r] = (p >= 0 && p < sd.n_vis) ? p : -1;
            }
        }
        // delta = (position inside the sequence) - (rank among the sequence's kept rows)
        int seq_lo = first_lo, seq_kept = first_kept;
        if (sd.seq_offsets != nullptr) {
            int b = b_first;
            while (b + 1 < sd.B && sd.seq_offsets[b + 1] <= pos) ++b;
            if (b != b_first) {                  // the sequence starts inside this word
                seq_lo = min(max(sd.seq_offsets[b], word_pos + 1), word_pos + kMaskWord - 1);
                seq_kept = base + __popc(mask & ((1u << (seq_lo - word_pos)) - 1u));
            }
        }
        // 0 <= delta < S <= rope_len for well-formed offsets; clamped so that no table row outside is read
        const int delta = min(max((pos - seq_lo) - (base + r - seq_kept), 0), rope_len - 1);
        const float* ct = rope_cos + (size_t)delta * half;
        const float* st = rope_sin + (size_t)delta * half;
        // table entries of this thread's pairs: LAYOUT 0: pairs q*E .. q*E+E-1 (x in piece q, y in piece
        // q+hp); LAYOUT 1: piece q holds pairs q*E/2 .., piece q+hp holds pairs (q+hp)*E/2 ..
        float c[E], sn[E];
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int i = LAYOUT == 0 ? q * E + e : (e < E / 2 ? q * (E / 2) + e : (q + hp) * (E / 2) + (e - E / 2));
            c[e] = ct[i];
            sn[e] = st[i];
        }
        const long long src_off = (long long)pos * stride_s_bytes + (long long)q * 16;
        const long long dst_off = (long long)(base + r) * row_bytes + (long long)q * 16;
        const long long hop = (long long)hp * 16;
        constexpr int kHeads = CH > 0 ? (CH < 4 ? CH : 4) : 2;          // heads per batch (4 loads each)
        const int h_begin = CH > 0 ? 0 : (int)blockIdx.y * kHeads;
        const int h_end = CH > 0 ? H : (h_begin + kHeads < H ? h_begin + kHeads : H);
        for (int h0 = h_begin; h0 < h_end; h0 += kHeads) {
            uint4 kx[kHeads], ky[kHeads], vx[kHeads], vy[kHeads];
#pragma unroll
            for (int k = 0; k < kHeads; ++k) {
                int h = h0 + k;
                if (CH == 0) h = h < H ? h : H - 1;                     // a valid head, loaded twice
                const char* pk = K + h * stride_h_bytes + src_off;
                const char* pv = V + h * stride_h_bytes + src_off;
                kx[k] = load_stream(reinterpret_cast<const uint4*>(pk));
                ky[k] = load_stream(reinterpret_cast<const uint4*>(pk + hop));
                vx[k] = load_stream(reinterpret_cast<const uint4*>(pv));
                vy[k] = load_stream(reinterpret_cast<const uint4*>(pv + hop));
            }
#pragma unroll
            for (int k = 0; k < kHeads; ++k) {
                const int h = h0 + k;
                if (CH == 0 && h >= H) continue;
                float a[E], b[E], an[E], bn[E];
                Piece<T>::widen(kx[k], a);
                Piece<T>::widen(ky[k], b);
                if (LAYOUT == 0) {
#pragma unroll
                    for (int e = 0; e < E; ++e) rotate_back(a[e], b[e], c[e], sn[e], &an[e], &bn[e]);
                } else {
#pragma unroll
                    for (int e = 0; e < E / 2; ++e) {
                        rotate_back(a[2 * e], a[2 * e + 1], c[e], sn[e], &an[2 * e], &an[2 * e + 1]);
                        rotate_back(b[2 * e], b[2 * e + 1], c[E / 2 + e], sn[E / 2 + e], &bn[2 * e], &bn[2 * e + 1]);
                    }
                }
                char* ok = K_out + h * out_stride_h_bytes + dst_off;
                char* ov = V_out + h * out_stride_h_bytes + dst_off;
                store_stream(reinterpret_cast<uint4*>(ok), Piece<T>::narrow(an));
                store_stream(reinterpret_cast<uint4*>(ok + hop), Piece<T>::narrow(bn));
                store_stream(reinterpret_cast<uint4*>(ov), vx[k]);
                store_stream(reinterpret_cast<uint4*>(ov + hop), vy[k]);
            }
        }
    }
}

template <typename T, int LAYOUT>
static void launch_kv_gather_rope(const KvArgs& a, const uint16_t* mask16, const int32_t* word_base, int n_words,
                                  size_t esz) {
#define SHARPV_GATHER_ROPE(CH_)                                                                                     \
    hipLaunchKernelGGL((kv_gather_rope_kernel<T, LAYOUT, CH_>), dim3(n_words + a.B, CH_ > 0 ? 1 : (a.H + 1) / 2),     \
                       dim3(kGatherThreads), 0,                                                                      \
                       a.stream, (const char*)a.K, (const char*)a.V, (long long)(a.kv_stride_h * (int64_t)esz),     \
                       (long long)(a.kv_stride_s * (int64_t)esz), (char*)a.K_out, (char*)a.V_out,                    \
                       (long long)(a.out_stride_h * (int64_t)esz), (int)(a.D * esz), a.H, mask16, word_base, n_words,\
                       a.sd, a.S, a.out_idx, a.out_count, a.out_orig_row, a.rope_cos, a.rope_sin, a.rope_len)
    switch (a.H) {
        case 2: SHARPV_GATHER_ROPE(2); break;
        case 4: SHARPV_GATHER_ROPE(4); break;
        case 8: SHARPV_GATHER_ROPE(8); break;
        default: SHARPV_GATHER_ROPE(0);
    }
#undef SHARPV_GATHER_ROPE
}

// ---------------------------------------------------------------------------- host side
int launch_prune_kv(const KvArgs& a) {
    hipStream_t st = a.stream;
    const int n_groups = (a.S + kGroup - 1) / kGroup;
    KvWorkspace ws = carve_kv_workspace(a.workspace, a.B, a.S, a.sd.orig_row != nullptr ? a.S : a.n_vis);
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
    const int32_t* word_base = nullptr;
    if (n_words > kGatherSelfScanWords) {
        TimedLaunch tl(kKvMaskScan, st);
        hipLaunchKernelGGL(kv_mask_scan_kernel, dim3(1), dim3(1024), 0, st, mask16, n_words, ws.word_base);
        word_base = ws.word_base;
        if (hipGetLastError() != hipSuccess) return SHARPV_ERR_DEVICE;
    }
    if (a.rope_cos != nullptr) {
        TimedLaunch tl(kKvGatherRope, st);
        if (a.dtype == SHARPV_BF16) {
            if (a.rope_layout == 0) launch_kv_gather_rope<bf16_t, 0>(a, mask16, word_base, n_words, esz);
            else launch_kv_gather_rope<bf16_t, 1>(a, mask16, word_base, n_words, esz);
        } else {
            if (a.rope_layout == 0) launch_kv_gather_rope<float, 0>(a, mask16, word_base, n_words, esz);
            else launch_kv_gather_rope<float, 1>(a, mask16, word_base, n_words, esz);
        }
    } else {
        TimedLaunch tl(kKvGather, st);
#define SHARPV_GATHER(CH_)                                                                                          \
    hipLaunchKernelGGL((kv_gather_kernel<CH_>),                                                                     \
                       dim3(n_words + a.B, CH_ > 0 ? 1 : (2 * a.H + kGatherBatch - 1) / kGatherBatch),                 \
                       dim3(kGatherThreads), 0, st, (const char*)a.K, (const char*)a.V, (long long)(a.kv_stride_h * (int64_t)esz),                                  \
                       (long long)(a.kv_stride_s * (int64_t)esz), (char*)a.K_out, (char*)a.V_out,                    \
                       (long long)(a.out_stride_h * (int64_t)esz), (int)(a.D * esz), a.H, mask16, word_base, n_words,\
                       a.sd, a.S, a.out_idx, a.out_count, a.out_orig_row)
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
