// Pre-LLM stage (Sec. 3.1, Eq.1-6): frame means, per-token inner products, dissimilarities and
// scores, per-frame retention ratio and top-k, and the compaction of the token stream.
//
// Kernels
//   frame_slab    (bf16, f <= 208) fused first two steps with every feature read once: a workgroup owns
//                 one 256-column slab (= one block of the summation order) and walks a run of consecutive
//                 frames with two frame slabs packed in registers (the frame that arrives and the one before
//                 it, whose registers are refilled row by row with the frame after).  One pass per frame
//                 widens both once: column sums by row class -> LDS -> halving tree -> slab of the frame
//                 mean, the slab's share of x.x and x.x_prev per row, and the share of x.mean of the frame
//                 before.  The per-slab shares are summed in ascending slab order by frame_select.
//   frame_mean    (other shapes) workgroup = (frame, 256-column slab), 32 row classes x 32 lanes: row i goes to
//                 class i % 32, each class adds its rows in ascending order (eight streamed loads issued
//                 before their sums), the 32 classes are reduced by a halving tree in LDS, divided by f.
//                 Eq.2's average representation.
//   token_dots    one wavefront per (token slot, run of frames): x.x, x.mean_t and x.x_prev in the fixed
//                 order of sharpv_device.hpp.  The slot's row of frame t stays in registers as x_prev of
//                 frame t+1 while the row of frame t+1 streams in, the frame mean is staged in LDS, so
//                 this pass reads the features once more and no more than that.
//   frame_select  one workgroup per frame: Eq.1-4 from the stored inner products, Eq.5/6 retention ratio
//                 and kept count, rank of every token by counting 64-bit keys (score descending, index
//                 ascending) staged in LDS, and the frame's kept rows in ascending order.
//   token_gather  copies the kept rows into the compacted stream and writes their indices, one
//                 wavefront per kept row; every workgroup scans the per-frame counts itself.
//   count_scan    exclusive scan of the per-frame kept counts, only for batches of more frames than
//                 token_gather stages in LDS.
#include <type_traits>
#include "sharpv_kernels.hpp"

namespace sharpv {

static int num_compute_units();

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
        // rows g, g+32, ... in ascending order, eight loads issued before their sums (clamped row index:
        // no load under a predicate)
        const T* col = feats + (size_t)t * f * d + (size_t)c * kChunk;
        const int mine = f > g ? (f - g + 31) / 32 : 0;
        for (int j0 = 0; j0 < mine; j0 += 8) {
            RawChunk<T> r[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int i = g + 32 * (j0 + j);
                r[j] = load_raw_stream<T>(col + (size_t)(i < f ? i : f - 1) * d);
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (j0 + j < mine) {
                    float v[8];
                    unpack(r[j], v);
#pragma unroll
                    for (int k = 0; k < 8; ++k) p[k] = p[k] + v[k];
                }
            }
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

// ---------------------------------------------------------------------------- fused mean + inner products
constexpr int kSlabThreads = 512;   // 16 row groups x 32 lanes

// A workgroup owns slab `slab` (256 columns = one block of the summation order) of the frames
// [t0, t1) and walks them in order.  Thread (g, l): lane l owns chunk l of the slab, row group g owns
// rows g, g+16, g+32, ... of a frame (KR = ceil(f/16) rows per thread, so only the last of them can
// fall outside the frame).  Row i belongs to class i % 32 of the column sum, i.e. class g for even k
// and class g+16 for odd k (i = g + 16k).
//
// Two frame slabs live in registers as packed bf16: the frame that has just arrived (`curr`, frame
// t) and the one before it (`prev`).  One pass over the thread's rows widens each of them once and
// takes everything that needs them: the column sums of frame t, the slab's shares of x.x and
// x.x_prev of frame t, and the share of x.mean of frame t-1, whose mean slab was finished at the end
// of the previous step.  As soon as a row of `prev` has been widened its registers receive the same
// row of frame t+1, so those loads are in flight for a whole step.  The two buffers swap roles from
// step to step.
//
// A run starts with its own first frame and no predecessor, so its first loads are ones it needs
// anyway.  x.x_prev of that frame is made where its predecessor already sits in registers: by the
// run before it (same slab, ending at t1 = this run's t0), which after its last frame takes one more,
// shorter step on frame t1 (x.x_prev of frame t1 and x.mean of frame t1-1, nothing else).  A run that
// ends with the sequence takes x.mean of its last frame alone.
//
// Every lane loads from a valid address (row and chunk indices are clamped) so that no load sits
// under a per-lane predicate; lanes past the end of a row contribute zeros to the trees, and the
// one row per thread that may lie past the frame is zeroed before it enters the column sums.
constexpr int kSlabRowLds = kBlockElems + kBlockChunks;   // a 256-column row in LDS plus its pad words
constexpr int kSlabWindow = 16;                           // frames whose shares wait in LDS before they are written
constexpr int kSlabStage = kSlabWindow * 208 + 64;        // a window of frames (f <= 208) plus the row slots past the last
constexpr int kSlabStageTotal = 256 + 3 * kSlabStage;     // a spare row, then x.x, x.x_prev, x.mean

//
// A workgroup whose share crosses into the next slab would stop in mid-work to wait for two fresh frame
// slabs, and finish that much later than the others.  So the buffers belong to the workgroup, not to
// the run: where a run ends with the sequence, another run follows in the same workgroup, the last
// frame sits in A (an even number of frames) and the next slab has all its columns, the last step's
// refill of B (which past the sequence's end would fetch nothing of use) takes frame 0 of the next
// slab, 32 chunks further along the same rows.  The run then returns true, and the run that follows
// is one that finds B on its way (PRELOADED) and asks only for A.
template <int KR, bool PRELOADED>
__device__ __forceinline__ bool slab_run(const bf16_t* __restrict__ feats, const int n, const int f, const int d,
                                         const int nslabs, const int slab, const int t0, const int t1,
                                         float* __restrict__ part_aa, float* __restrict__ part_am,
                                         float* __restrict__ part_ab, float* __restrict__ part_mm,
                                         float (&sm)[16][kSlabRowLds], float (&smean)[kSlabRowLds],
                                         float (&sstage)[kSlabStageTotal], RawChunk<bf16_t> (&A)[KR],
                                         RawChunk<bf16_t> (&B)[KR], const bool run_follows) {
    // Opaque to the compiler, so that what a run derives from the thread index is derived anew by
    // every run: hoisted out of the caller's loop over runs, those values would stay alive through the
    // steps next to the two buffers, beyond the register file.
    int tid_opaque = threadIdx.x;
    asm volatile("" : "+v"(tid_opaque));
    const int tid = tid_opaque;
    const int l = tid & 31;
    const int g = tid >> 5;
    const int nchunks = d / kChunk;
    const int c = slab * kBlockChunks + l;
    const bool live = c < nchunks;
    const size_t N = (size_t)n * f;
    const size_t frame_bytes = (size_t)f * d * sizeof(bf16_t);
    const char* const fbase = reinterpret_cast<const char*>(feats);
    const uint32_t chunk_off = (uint32_t)((live ? c : nchunks - 1) * kChunk * (int)sizeof(bf16_t));
    const uint32_t row_bytes = (uint32_t)d * (uint32_t)sizeof(bf16_t);
    uint32_t off[KR];                            // byte offsets of the thread's chunks inside a frame
#pragma unroll
    for (int k = 0; k < KR; ++k) {
        const int i = g + 16 * k;
        off[k] = (uint32_t)(i < f ? i : f - 1) * row_bytes + chunk_off;
    }
    const bool last_row_valid = g + 16 * (KR - 1) < f;

    // tree32_quad(a, b, c, d) leaves a, c, b, d in lanes 7, 15, 23, 31 of a half-wavefront; this
    // lane's quarter decides which result it stores and where.
    const int quarter = l >> 3;
    const bool qlead = (l & 7) == 7;
    // (x.x, x.x_prev) of rows k and k+1 -> quarters 0..3 hold aa[k], aa[k+1], ab[k], ab[k+1]
    const int pair_row = quarter & 1;
    const bool pair_is_ab = (quarter & 2) != 0;
    float* const pair_ptr = (pair_is_ab ? part_ab : part_aa) + (size_t)slab * N + g + 16 * pair_row;
    // x.mean of rows k .. k+3 -> quarters 0..3 hold am[k], am[k+2], am[k+1], am[k+3]
    const int mean_row = (quarter & 1) * 2 + (quarter >> 1);
    float* const mean_ptr = part_am + (size_t)slab * N + g + 16 * mean_row;
    // Where the same values wait in LDS: the shares of a window of frames are kept there and written
    // out together (see flush below).  Lanes that hold no result write to a spare row, so that these
    // writes need no lane mask.  Slot j of the window is frame w0 + j for x.x and x.x_prev and frame
    // w0 + j - 1 for x.mean (which a step makes one frame late).
    const int stage_arr = 256 + (pair_is_ab ? kSlabStage : 0);
    const int stage_pair0 = qlead ? stage_arr + g + 16 * pair_row : g;
    const int stage_last0 = qlead && pair_row == 0 ? stage_arr + g : g;
    const int stage_mean0 = qlead ? 256 + 2 * kSlabStage + g + 16 * mean_row : g;
    const int stage_step = qlead ? f : 0;        // the spare row does not move with the window slot
    const int stage_last_step = qlead && pair_row == 0 ? f : 0;
    int w0 = t0;                                 // first frame of the window
    int wj = 0;                                  // frames in the window so far
    float* stage_pair = sstage + stage_pair0;
    float* stage_last = sstage + stage_last0;
    float* stage_mean = sstage + stage_mean0;

    // Writes the window's shares to memory, whole lines at a time, and starts the next window.  Every
    // staging write of the window lies before a barrier of the column phase that all threads have
    // passed.  In the first window of a run, slot 0 holds no x.x_prev (the run before makes it) and no
    // x.mean (there is no earlier frame here).
    auto flush = [&]() {
        const int cnt = wj * f;
        const int lo = w0 == t0 ? f : 0;
        const size_t base = (size_t)slab * N + (size_t)w0 * f;
        for (int i = tid; i < cnt; i += kSlabThreads) {
            part_aa[base + i] = sstage[256 + i];
            if (i >= lo) {
                part_ab[base + i] = sstage[256 + kSlabStage + i];
                part_am[base + i - f] = sstage[256 + 2 * kSlabStage + i];
            }
        }
        __syncthreads();                         // before the slots are written again
        w0 += wj;
        wj = 0;
        stage_pair = sstage + stage_pair0;
        stage_last = sstage + stage_last0;
        stage_mean = sstage + stage_mean0;
    };

    // Trees and stores of the x.mean shares of frame tm (four rows per tree, zero padding at the end).
    // staged = true: into the workgroup's staging rows (written out in whole lines during the column
    // phase); staged = false: straight to memory.
    auto mean_products = [&](const float (&am)[KR], const int tm, auto staged_c) {
        constexpr bool staged = decltype(staged_c)::value;
        float* const pm = mean_ptr + (size_t)tm * f;
#pragma unroll
        for (int k = 0; k < KR; k += 4) {
            const float z = tree32_quad(am[k], k + 1 < KR ? am[k + 1] : 0.0f, k + 2 < KR ? am[k + 2] : 0.0f,
                                        k + 3 < KR ? am[k + 3] : 0.0f);
            const int r = k + mean_row;          // this lane's row slot
            if constexpr (staged) {
                stage_mean[16 * k] = z;
            } else {
                const bool ok = (k + 3 < KR - 1) || (r < KR - 1) || (r == KR - 1 && last_row_valid);
                if (qlead && ok) pm[16 * k] = z;
            }
        }
    };

    float m[8];                                  // this lane's chunk of the latest frame-mean slab
#pragma unroll
    for (int j = 0; j < 8; ++j) m[j] = 0.0f;

    const bool extra = t1 < n;                   // this run also makes x.x_prev of the next run's first frame
    // what a refill past the sequence's end fetches: frame 0 of the next slab, else the last frame again
    const bool hand_over = !PRELOADED && run_follows && !extra && ((t1 - t0) & 1) == 0 &&
                           (slab + 2) * kBlockChunks <= nchunks;
    const char* const past_end = hand_over ? fbase + (size_t)kBlockChunks * kChunk * sizeof(bf16_t)
                                           : fbase + (size_t)(n - 1) * frame_bytes;
    auto step = [&](RawChunk<bf16_t> (&prev)[KR], RawChunk<bf16_t> (&curr)[KR], const int t, auto with_prev_c,
                    auto curr_stats_c) {
        constexpr bool with_prev = decltype(with_prev_c)::value;       // false: the run's first frame
        constexpr bool curr_stats = decltype(curr_stats_c)::value;     // false: the extra step (frame t1)
        // A full step always refills (past the sequence's end: see past_end), so that the loads sit under
        // no condition.
        constexpr bool has_next = with_prev && curr_stats;
        const bool store_ab = with_prev && t > 0;
        const char* const nb = t + 1 < n ? fbase + (size_t)(t + 1) * frame_bytes : past_end;
        float* const pp = pair_ptr + (size_t)t * f;
        // column sums: rows of class g (even k) and class g+16 (odd k), each ascending; the
        // stride-16 level of the class tree adds the two right here
        float pe[8], po[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) { pe[j] = 0.0f; po[j] = 0.0f; }
        float am[KR];
        float zq[(KR + 1) / 2];
        float aa_even = 0.0f, ab_even = 0.0f;
        // keep "uniform frame base + 32-bit lane offset" addressing: without this the lane offsets are
        // widened and added to the feature pointer once, outside the loop, at two registers per row
#pragma unroll
        for (int k = 0; k < KR; ++k) asm volatile("" : "+v"(off[k]));
#pragma unroll
        for (int k = 0; k < KR; ++k) {
            if (k == KR - 1) {                   // the only row that can lie past the frame
                curr[k].q.x = last_row_valid ? curr[k].q.x : 0u;
                curr[k].q.y = last_row_valid ? curr[k].q.y : 0u;
                curr[k].q.z = last_row_valid ? curr[k].q.z : 0u;
                curr[k].q.w = last_row_valid ? curr[k].q.w : 0u;
            }
            float a[8], b[8];
            unpack(curr[k], a);
            if constexpr (with_prev) unpack(prev[k], b);
            if constexpr (curr_stats) {
                if (k & 1) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) po[j] = po[j] + a[j];
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j) pe[j] = pe[j] + a[j];
                }
            }
            float vaa = 0.0f, vab = 0.0f, vam = 0.0f;
            if constexpr (curr_stats) vaa = chain8(a, a);
            if constexpr (with_prev) { vab = chain8(a, b); vam = chain8(b, m); }
            if constexpr (has_next) prev[k].q = load_stream(reinterpret_cast<const uint4*>(nb + off[k]));
            vaa = live ? vaa : 0.0f;
            vab = live ? vab : 0.0f;
            am[k] = live ? vam : 0.0f;
            if (k & 1) {
                zq[k / 2] = tree32_quad(aa_even, ab_even, vaa, vab);
            } else if (k == KR - 1) {            // odd row count: the last row alone (quarters 0 and 2 store)
                zq[k / 2] = tree32_pair(vaa, vab);
            } else {
                aa_even = vaa;
                ab_even = vab;
            }
            // Pin the row's results here: everything that needs the widened rows is finished before
            // the next rows start, so their sixteen floats do not stay alive (the compiler otherwise
            // sinks the column sums and the x.mean chains to the end of the step).
            if (k & 1)
                asm volatile("" : "+v"(po[0]), "+v"(po[1]), "+v"(po[2]), "+v"(po[3]), "+v"(po[4]), "+v"(po[5]),
                                  "+v"(po[6]), "+v"(po[7]), "+v"(am[k]), "+v"(zq[k / 2]));
            else
                asm volatile("" : "+v"(pe[0]), "+v"(pe[1]), "+v"(pe[2]), "+v"(pe[3]), "+v"(pe[4]), "+v"(pe[5]),
                                  "+v"(pe[6]), "+v"(pe[7]), "+v"(am[k]));
            __builtin_amdgcn_sched_barrier(0);
        }
        // The shares leave the thread only now, after the refill loads.  A full step hands them to the
        // window in LDS: stores that mingle with the stream of loads, even as whole lines, cost several
        // microseconds per launch; one burst of stores per window (normally: per run) costs about half.
        const std::true_type staged{};
        const std::false_type direct{};
        if constexpr (curr_stats) {
#pragma unroll
            for (int k = 0; k < KR; ++k) {
                if (k & 1) {
                    stage_pair[16 * (k - 1)] = zq[k / 2];
                } else if (k == KR - 1) {
                    stage_last[16 * k] = zq[k / 2];
                }
            }
            if constexpr (with_prev) mean_products(am, t - 1, staged);
        } else {
#pragma unroll
            for (int k = 0; k < KR; ++k) {
                if (k & 1) {
                    const bool ok = (k < KR - 1) || pair_row == 0 || last_row_valid;
                    if (qlead && ok && pair_is_ab && store_ab) pp[16 * (k - 1)] = zq[k / 2];
                } else if (k == KR - 1) {
                    if (qlead && pair_row == 0 && last_row_valid && pair_is_ab && store_ab) pp[16 * k] = zq[k / 2];
                }
            }
            mean_products(am, t - 1, direct);
            return;
        }
        // The next step widens `curr` again (as its `prev`); make the compiler forget the widened
        // copies instead of keeping eight floats per chunk alive across the step boundary.
#pragma unroll
        for (int k = 0; k < KR; ++k)
            asm volatile("" : "+v"(curr[k].q.x), "+v"(curr[k].q.y), "+v"(curr[k].q.z), "+v"(curr[k].q.w));

#pragma unroll
        for (int j = 0; j < 8; ++j) sm[g][l * 9 + j] = pe[j] + po[j];
        __syncthreads();
        if (tid < kBlockElems) {                 // one thread per column: strides 8, 4, 2, 1 over the 16 sums
            float q[16];
#pragma unroll
            for (int gg = 0; gg < 16; ++gg) q[gg] = sm[gg][tid + (tid >> 3)];
#pragma unroll
            for (int st = 8; st >= 1; st >>= 1)
#pragma unroll
                for (int ll = 0; ll < st; ++ll) q[ll] = q[ll] + q[ll + st];
            smean[tid + (tid >> 3)] = q[0] / (float)f;
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 8; ++j) m[j] = smean[l * 9 + j];
        if (tid < 64) {                          // this slab's share of mean.mean
            const float mm = chain8(m, m);
            const float v = tree32(live ? mm : 0.0f);
            if (tid == 0) part_mm[(size_t)t * nslabs + slab] = v;
        }
        ++wj;
        stage_pair += stage_step;
        stage_last += stage_last_step;
        stage_mean += stage_step;
        if (wj == kSlabWindow) flush();
    };

    // x.mean of the sequence's last frame, still packed in `buf`, against the mean slab just finished
    auto tail = [&](const RawChunk<bf16_t> (&buf)[KR], const int t) {
        float am[KR];
#pragma unroll
        for (int k = 0; k < KR; ++k) {
            float b[8];
            unpack(buf[k], b);
            const float vam = chain8(b, m);
            am[k] = live ? vam : 0.0f;
        }
        mean_products(am, t, std::false_type{});
    };

    {
        const char* const b1 = fbase + (size_t)t0 * frame_bytes;
        const char* const b2 = fbase + (size_t)(t0 + 1 < n ? t0 + 1 : n - 1) * frame_bytes;
        if constexpr (!PRELOADED) {
#pragma unroll
            for (int k = 0; k < KR; ++k) B[k].q = load_stream(reinterpret_cast<const uint4*>(b1 + off[k]));
        }
#pragma unroll
        for (int k = 0; k < KR; ++k) A[k].q = load_stream(reinterpret_cast<const uint4*>(b2 + off[k]));
    }
    const std::true_type yes{};
    const std::false_type no{};
    step(A, B, t0, no, yes);                     // the run's first frame: no predecessor here
    int t = t0 + 1;
    for (; t + 1 < t1; t += 2) {
        step(B, A, t, yes, yes);                 // prev = B, curr = A; B is refilled with frame t+1
        step(A, B, t + 1, yes, yes);
    }
    if (t < t1) {
        step(B, A, t, yes, yes);
        if (extra) step(A, B, t1, yes, no); else tail(A, t1 - 1);
    } else {
        if (extra) step(B, A, t1, yes, no); else tail(B, t1 - 1);
    }
    if (wj > 0) flush();
    return hand_over;
}

// The (slab, frame) pairs, slab-major, are dealt out in equal contiguous runs, one per workgroup
// (about one workgroup per compute unit): a run that crosses into the next slab continues there at
// frame 0, which has no predecessor, so every workgroup reads at most one frame slab beyond its
// own share (the first frame of the run that follows, at the very end).
template <int KR>
__global__ __launch_bounds__(kSlabThreads) void frame_slab_kernel(const bf16_t* __restrict__ feats, int n, int f, int d,
                                                                  int nslabs, int run_len, int run_extra,
                                                                  float* __restrict__ part_aa,   // [nslabs][n*f]
                                                                  float* __restrict__ part_am,
                                                                  float* __restrict__ part_ab,
                                                                  float* __restrict__ part_mm) { // [n][nslabs]
    // column c sits at index c + c/8 (one pad word per chunk of 8), which spreads a lane's 8
    // consecutive words and the other lanes' over distinct LDS banks
    __shared__ float sm[16][kSlabRowLds];        // column sums of classes g and g+16 already added
    __shared__ float smean[kSlabRowLds];
    __shared__ float sstage[kSlabStageTotal];    // a window of frames' x.x, x.x_prev, x.mean shares on their way out
    // runs of run_len pairs, the first run_extra of them one pair longer
    const int w = blockIdx.x;
    long long u = (long long)w * run_len + (w < run_extra ? w : run_extra);   // nslabs * n may pass 2^31
    const long long u_end = u + run_len + (w < run_extra ? 1 : 0);
    int slab = (int)(u / n);
    int t0 = (int)(u - (long long)slab * n);
    long long left = u_end - u;                  // pairs still to do; every run after the first starts a slab
    RawChunk<bf16_t> A[KR], B[KR];               // the two frame slabs in flight (see slab_run)
    while (left > 0) {
        int t1 = (long long)t0 + left < n ? t0 + (int)left : n;
        left -= t1 - t0;
        const bool handed = slab_run<KR, false>(feats, n, f, d, nslabs, slab, t0, t1, part_aa, part_am, part_ab,
                                                  part_mm, sm, smean, sstage, A, B, left > 0);
        ++slab;
        t0 = 0;
        if (handed) {                            // the next run finds its first frame on its way
            t1 = left < n ? (int)left : n;
            left -= t1;
            slab_run<KR, true>(feats, n, f, d, nslabs, slab, 0, t1, part_aa, part_am, part_ab, part_mm, sm, smean,
                               sstage, A, B, false);
            ++slab;
        }
    }
}

// ---------------------------------------------------------------------------- per-token inner products
// One token row as a wavefront holds it: chunk c = 64*q + lane in sweep q.  NS = number of sweeps
// (d <= 512*NS); FULL = every lane of every sweep holds a chunk (d == 512*NS).
template <typename T, int NS> struct RowRegs { RawChunk<T> r[NS]; };

template <typename T, int NS, bool FULL, bool STREAM>
__device__ __forceinline__ void load_row(const T* __restrict__ row, int nchunks, int lane, RowRegs<T, NS>& out) {
#pragma unroll
    for (int q = 0; q < NS; ++q) {
        const int c = q * 64 + lane;
        // lanes past the end of the row reload its last chunk (no load under a predicate); they are
        // masked out of the sums
        const T* p = row + (size_t)(FULL || c < nchunks ? c : nchunks - 1) * kChunk;
        out.r[q] = STREAM ? load_raw_stream<T>(p) : load_raw<T>(p);
    }
}

// Any d: sweeps in a loop, straight from memory (rows wider than the unrolled sweeps cover).
template <typename T>
__device__ __forceinline__ void row_dots_loop(const T* __restrict__ x, const T* __restrict__ xp,
                                              const float* __restrict__ m, int nchunks, int lane,
                                              float* s_aa, float* s_am, float* s_ab) {
    float aa = 0.0f, am = 0.0f, ab = 0.0f;
    for (int c0 = 0; c0 < nchunks; c0 += 64) {
        const int c = c0 + lane;
        float paa = 0.0f, pam = 0.0f, pab = 0.0f;
        if (c < nchunks) {
            float a[8], b[8], mm[8];
            unpack(load_raw<T>(x + (size_t)c * kChunk), a);
            unpack(load_raw<T>(xp + (size_t)c * kChunk), b);
            unpack(load_raw<float>(m + (size_t)c * kChunk), mm);
            paa = chain8(a, a);
            pam = chain8(a, mm);
            pab = chain8(a, b);
        }
        paa = tree32(paa);
        pam = tree32(pam);
        pab = tree32(pab);
        const bool odd = c0 + kBlockChunks < nchunks;
        aa = add_blocks(aa, paa, odd);
        am = add_blocks(am, pam, odd);
        ab = add_blocks(ab, pab, odd);
    }
    *s_aa = aa; *s_am = am; *s_ab = ab;
}

// One wavefront per (token slot, run of consecutive frames), four slots per workgroup, all four on the same
// run.  The wavefront walks its slot through the frames of the run with two row buffers in registers: the
// row of frame t and the row of frame t-1; sweep by sweep, as soon as a chunk of the older row has been
// widened its registers receive the same chunk of frame t+1, so a whole row of loads is in flight per
// wavefront while it works, and every feature is read once (plus one row per run, the predecessor of the
// run's first frame).  The feature rows are streamed (non-temporal).  The frame mean, which the four slots
// share, is staged in LDS one frame ahead (two planes of 16-byte pieces, so that a wavefront's reads meet
// no bank twice).
template <typename T, int NS, bool FULL>
__global__ __launch_bounds__(256) void token_dots_kernel(const T* __restrict__ feats, const float* __restrict__ mean,
                                                         int n, int f, int d, int run_len, int slot_blocks,
                                                         float* __restrict__ aa, float* __restrict__ am,
                                                         float* __restrict__ ab) {
    constexpr int kPieces = NS * 64;             // chunks a row can have at most
    __shared__ float4 smean[2][2][kPieces];      // [frame parity][low / high half of a chunk][chunk]
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int ib = blockIdx.x % slot_blocks;
    const int run = blockIdx.x / slot_blocks;
    const int t0 = run * run_len;
    if (t0 >= n) return;                         // whole workgroup
    const int t1 = t0 + run_len < n ? t0 + run_len : n;
    const int slot_i = ib * 4 + (tid >> 6);
    const bool active = slot_i < f;              // a wavefront past the last slot still takes part in staging and barriers
    const int i = active ? slot_i : f - 1;
    const int nchunks = d / kChunk;
    const size_t frame_elems = (size_t)f * d;
    const T* const slot = feats + (size_t)i * d;                       // row i of frame 0

    // mean row of frame t -> LDS buffer `par`: float4 piece v of the row is half v % 2 of chunk v / 2
    constexpr int kStage = (2 * kPieces + 255) / 256;   // at most 4: 16-byte pieces of a mean row per thread
    static_assert(kStage <= 4, "unrolled sweeps cover rows of up to 4096 elements");

    // One frame: sums of row `cur` (frame t) against row `prev` (frame t-1) and the staged mean of frame
    // t; the registers of `prev` are refilled with the row of frame t+1.
    auto step = [&](RowRegs<T, NS>& prev, const RowRegs<T, NS>& cur, const int t) {
        const int tn = t + 1 < n ? t + 1 : n - 1;                      // clamped: always a valid load
        // (named registers, not an array: the stores further down sit under conditions, and an array would be
        // indexed in memory)
        const float4* mrow = reinterpret_cast<const float4*>(mean + (size_t)tn * d);
        const int last_piece = 2 * nchunks - 1;
        auto piece = [&](int k) { const int v = tid + 256 * k; return mrow[v < last_piece ? v : last_piece]; };
        float4 st0 = piece(0), st1, st2, st3;
        if constexpr (kStage > 1) st1 = piece(1);
        if constexpr (kStage > 2) st2 = piece(2);
        if constexpr (kStage > 3) st3 = piece(3);
        const T* const next_row = slot + (size_t)tn * frame_elems;
        const int par = t & 1;
        float s_aa = 0.0f, s_am = 0.0f, s_ab = 0.0f;
#pragma unroll
        for (int q = 0; q < NS; ++q) {
            const int c = q * 64 + lane;
            const bool have = FULL || c < nchunks;
            const int cc = have ? c : nchunks - 1;
            float a[8], b[8], mm[8];
            unpack(cur.r[q], a);
            unpack(prev.r[q], b);
            prev.r[q] = load_raw_stream<T>(next_row + (size_t)cc * kChunk);
            const float4 lo = smean[par][0][cc], hi = smean[par][1][cc];
            mm[0] = lo.x; mm[1] = lo.y; mm[2] = lo.z; mm[3] = lo.w;
            mm[4] = hi.x; mm[5] = hi.y; mm[6] = hi.z; mm[7] = hi.w;
            const float vaa = have ? chain8(a, a) : 0.0f;
            const float vam = have ? chain8(a, mm) : 0.0f;
            const float vab = have ? chain8(a, b) : 0.0f;
            const float pair = tree32_pair(vaa, vam);                  // rows 0,2: x.x   rows 1,3: x.mean
            const float single = tree32(vab);
            const bool odd = FULL || (q * 64 + kBlockChunks < nchunks); // does the sweep's second block exist
            s_aa = s_aa + lane_value(pair, 0);
            s_am = s_am + lane_value(pair, 16);
            s_ab = s_ab + lane_value(single, 0);
            if (odd) {
                s_aa = s_aa + lane_value(pair, 32);
                s_am = s_am + lane_value(pair, 48);
                s_ab = s_ab + lane_value(single, 32);
            }
            __builtin_amdgcn_sched_barrier(0);   // one sweep at a time: keeps the widened copies of one chunk alive, not of all
        }
        if (lane == 0 && active) {
            const size_t row = (size_t)t * f + i;
            aa[row] = s_aa;
            am[row] = s_am;
            ab[row] = t > 0 ? s_ab : 0.0f;
        }
        // nobody reads the other buffer any more: its frame ended at the last barrier
        auto put = [&](int k, const float4& v4) {
            const int v = tid + 256 * k;
            if (v <= last_piece) smean[par ^ 1][v & 1][v >> 1] = v4;
        };
        put(0, st0);
        if constexpr (kStage > 1) put(1, st1);
        if constexpr (kStage > 2) put(2, st2);
        if constexpr (kStage > 3) put(3, st3);
        __syncthreads();
    };

    RowRegs<T, NS> A, B;
    load_row<T, NS, FULL, true>(slot + (size_t)(t0 > 0 ? t0 - 1 : 0) * frame_elems, nchunks, lane, A);
    load_row<T, NS, FULL, true>(slot + (size_t)t0 * frame_elems, nchunks, lane, B);
    {
        const float4* mrow = reinterpret_cast<const float4*>(mean + (size_t)t0 * d);
        for (int v = tid; v < 2 * nchunks; v += 256) smean[t0 & 1][v & 1][v >> 1] = mrow[v];
    }
    __syncthreads();
    int t = t0;
    for (; t + 1 < t1; t += 2) {
        step(A, B, t);                           // prev = A, cur = B; A receives frame t+1
        step(B, A, t + 1);
    }
    if (t < t1) step(A, B, t);
}

// Rows wider than the unrolled sweeps cover: one wavefront per row, straight from memory.
template <typename T>
__global__ __launch_bounds__(256) void token_dots_wide_kernel(const T* __restrict__ feats, const float* __restrict__ mean,
                                                              int n_rows, int f, int d,
                                                              float* __restrict__ aa, float* __restrict__ am,
                                                              float* __restrict__ ab) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= n_rows) return;
    const int t = row / f;
    const T* x = feats + (size_t)row * d;
    const T* xp = t > 0 ? x - (size_t)f * d : x;
    float s_aa, s_am, s_ab;
    row_dots_loop<T>(x, xp, mean + (size_t)t * d, d / kChunk, lane, &s_aa, &s_am, &s_ab);
    if (lane == 0) {
        aa[row] = s_aa;
        am[row] = s_am;
        ab[row] = t > 0 ? s_ab : 0.0f;
    }
}

template <typename T>
static void launch_token_dots(const TokArgs& a, const TokWorkspace& ws) {
    const int nchunks = a.d / kChunk;
    const int ns = (nchunks + 63) / 64;
    const bool full = nchunks == ns * 64;
    const int slot_blocks = (a.f + 3) / 4;
    // enough wavefronts to fill the chip (about 16 per compute unit), runs as long as that allows
    const long long want_waves = 16ll * num_compute_units();
    long long runs = (want_waves + a.f - 1) / a.f;
    runs = runs < 1 ? 1 : (runs > a.n ? a.n : runs);
    const int run_len = (int)((a.n + runs - 1) / runs);
    const int n_runs = (a.n + run_len - 1) / run_len;
    const dim3 grid((unsigned)((long long)slot_blocks * n_runs)), block(256);
#define SHARPV_DOTS_CASE(NS_)                                                                                       \
    case NS_:                                                                                                       \
        if (full)                                                                                                   \
            hipLaunchKernelGGL((token_dots_kernel<T, NS_, true>), grid, block, 0, a.stream, (const T*)a.feats,      \
                               (const float*)ws.mean, a.n, a.f, a.d, run_len, slot_blocks, ws.aa, ws.am, ws.ab);    \
        else                                                                                                        \
            hipLaunchKernelGGL((token_dots_kernel<T, NS_, false>), grid, block, 0, a.stream, (const T*)a.feats,     \
                               (const float*)ws.mean, a.n, a.f, a.d, run_len, slot_blocks, ws.aa, ws.am, ws.ab);    \
        break;
    // float32 rows take twice the registers per sweep: four sweeps (d <= 2048) unrolled, wider rows loop
    switch (ns <= (sizeof(T) == 2 ? 8 : 4) ? ns : 0) {
        SHARPV_DOTS_CASE(1) SHARPV_DOTS_CASE(2) SHARPV_DOTS_CASE(3) SHARPV_DOTS_CASE(4)
        SHARPV_DOTS_CASE(5) SHARPV_DOTS_CASE(6) SHARPV_DOTS_CASE(7) SHARPV_DOTS_CASE(8)
        default:
            hipLaunchKernelGGL((token_dots_wide_kernel<T>), dim3((unsigned)(((long long)a.n * a.f + 3) / 4)), block, 0,
                               a.stream, (const T*)a.feats, (const float*)ws.mean, a.n * a.f, a.f, a.d, ws.aa, ws.am,
                               ws.ab);
    }
#undef SHARPV_DOTS_CASE
}

// ---------------------------------------------------------------------------- scores, ratio, top-k
// SB = share loads per array in flight per thread.  16 takes the 14 shares of the model width in one
// round trip but holds 64 loaded values (76 VGPRs: one 1024-thread workgroup per compute unit); 8 fits
// 64 VGPRs, so that two workgroups share a compute unit when there are more frames than compute units.
// The shares are added in ascending order either way.
template <int SB>
__global__ __launch_bounds__(1024, SB == 8 ? 8 : 4) void frame_select_kernel(const float* __restrict__ mean,      // [n][d] or nullptr
                                                            const float* __restrict__ part_mm,   // [n][nparts] if mean == nullptr
                                                            const float* __restrict__ aa, const float* __restrict__ am,
                                                            const float* __restrict__ ab,        // each [nparts][n*f]
                                                            int nparts, size_t part_stride,
                                                            const int32_t* __restrict__ frame_offsets, int B,
                                                            int f, int d, float w, int mode, float Kthr, int min_keep,
                                                            int measure,   // 0: Eq.1; 1: one minus cosine
                                                            int tpp,   // threads per copy of the frame (multiple of 64, >= f)
                                                            int32_t* __restrict__ local_idx,
                                                            int32_t* __restrict__ out_counts,
                                                            float* __restrict__ out_scores,
                                                            float* __restrict__ out_ratio) {
    __shared__ unsigned long long sKey[1024];    // (score as an ordered integer, inverted token index)
    __shared__ float sTT[1024];
    __shared__ float sblk[256];
    __shared__ float s_mm;
    __shared__ int s_first;
    __shared__ int s_k;
    __shared__ int wave_cnt[16];
    __shared__ int sRank[1024];

    // The workgroup holds blockDim.x / tpp copies of the frame's threads ("parts", whole wavefronts):
    // part 0 owns the tokens, the other parts only take a share of the ranking loop.
    const int t = blockIdx.x;
    const int tid = threadIdx.x;
    const int nthreads = blockDim.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int part = tid / tpp;
    const int parts = nthreads / tpp;
    const int nchunks = d / kChunk;
    const int nblocks = (nchunks + kBlockChunks - 1) / kBlockChunks;

    // Inner-product shares of this thread's token, summed in ascending block order (a single share
    // when the rows were summed whole).  The loads come first and in batches of SB shares x 4 arrays,
    // so that their latency overlaps the mean.mean and first-frame work below; indices are clamped
    // (no load under a predicate) and all four arrays are read whether or not the frame turns out to
    // be a first frame (x.x_prev of frame 0 is never written and never used).
    const int i = tid - part * tpp;
    const bool owner = part == 0 && i < f;
    const size_t r = (size_t)t * f + (i < f ? i : f - 1);
    const size_t rprev = t > 0 ? r - f : r;
    float xx = 0.0f, xm = 0.0f, xp = 0.0f, pp = 0.0f;
    if (nparts == 1 && part == 0) {
        xx = aa[r];
        xm = am[r];
        xp = ab[r];
        pp = aa[rprev];
    }
    for (int s0 = 0; nparts > 1 && part == 0 && s0 < nparts; s0 += SB) {
        float va[SB], vm[SB], vb[SB], vp[SB];
#pragma unroll
        for (int k = 0; k < SB; ++k) {
            const int sb = s0 + k < nparts ? s0 + k : nparts - 1;
            const size_t o = (size_t)sb * part_stride;
            va[k] = aa[o + r];
            vm[k] = am[o + r];
            vb[k] = ab[o + r];
            vp[k] = aa[o + rprev];
        }
#pragma unroll
        for (int k = 0; k < SB; ++k)
            if (s0 + k < nparts) {
                xx = xx + va[k];
                xm = xm + vm[k];
                xp = xp + vb[k];
                pp = pp + vp[k];
            }
    }

    // mean.mean in the common order: one half-wavefront per 256-element block (or the per-slab
    // shares left by the fused kernel)
    if (mean != nullptr) {
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
    } else {
        for (int b = tid; b < nblocks; b += nthreads) sblk[b] = part_mm[(size_t)t * nblocks + b];
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
    float score = 0.0f;
    if (owner) {
        const float S = measure_from_dots(measure, xm, xx, mm);              // Eq.2
        const float T = first ? S : measure_from_dots(measure, xp, xx, pp);  // Eq.3 (Eq.6 on a first frame)
        score = __builtin_fmaf(w, S, T);                                     // Eq.4
        // Ranking key: the float's bits mapped to an unsigned integer of the same order (inputs are
        // finite, and adding +0 folds -0 into +0 so that equal scores give equal keys), the inverted
        // index below it: key_j > key_i  <=>  token j is ahead of token i.
        const uint32_t ub = __float_as_uint(score + 0.0f);
        const uint32_t ord = (ub & 0x80000000u) ? ~ub : (ub | 0x80000000u);
        sKey[i] = ((unsigned long long)ord << 32) | (uint32_t)~(uint32_t)i;
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

    // top-k by counting: token i is kept iff fewer than k tokens are ahead of it (higher score, or
    // the same score and a lower index).  Each part counts over its slice of the frame.
    int rank = 0;
    if (mode == 0 && i < f) {
        const unsigned long long key = sKey[i];
        const int len = (f + parts - 1) / parts;
        const int j0 = part * len;
        const int j1 = j0 + len < f ? j0 + len : f;
#pragma unroll 8
        for (int j = j0; j < j1; ++j) rank += sKey[j] > key;
    }
    if (parts > 1) {
        sRank[tid] = rank;
        __syncthreads();
        if (part == 0)
            for (int q = 1; q < parts; ++q) rank += sRank[q * tpp + i];
    }
    int keep = 0;
    if (owner) keep = mode == 0 ? rank < s_k : score >= Kthr;
    const unsigned long long bal = __ballot(keep != 0);
    const int before = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0 && part == 0) wave_cnt[wave] = __popcll(bal);
    __syncthreads();
    int base = 0, total = 0;
    for (int q = 0; q < (tpp >> 6); ++q) {
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
    __shared__ int wave_tot[16];
    const int tid = threadIdx.x;
    const int seg = (n + 1023) / 1024;
    const int lo = tid * seg;
    const int hi = lo + seg < n ? lo + seg : n;
    int s = 0;
    for (int j = lo; j < hi; ++j) s += counts[j];
    const int incl = block_inclusive_scan_1024(s, wave_tot);
    int run = incl - s;                      // exclusive prefix of this thread's segment
    for (int j = lo; j < hi; ++j) {
        offsets[j] = run;
        run += counts[j];
    }
    if (tid == 1023) offsets[n] = incl;
}

// ---------------------------------------------------------------------------- compaction
// One wavefront per kept row j of the compacted stream: its frame is found by bisection of the
// offsets, its source row from the frame's kept list; out_feats[j] = feats[out_idx[j]].
// Up to kOffsetsInLds - 1 frames every workgroup builds the offsets itself from the per-frame counts
// (an exclusive scan in LDS; workgroup 0 also writes them out), which saves the scan kernel's launch;
// longer batches get the offsets from count_scan (counts == nullptr).
constexpr int kOffsetsInLds = 4096;
__global__ __launch_bounds__(256) void token_gather_kernel(const char* __restrict__ feats, int row_bytes, int n, int f,
                                                           const int32_t* __restrict__ counts,
                                                           int32_t* __restrict__ offsets,
                                                           const int32_t* __restrict__ local_idx,
                                                           int32_t* __restrict__ out_idx, char* __restrict__ out_feats) {
    __shared__ int soff[kOffsetsInLds];
    __shared__ int wave_tot[4];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const bool staged = counts != nullptr;       // host guarantees n + 1 <= kOffsetsInLds in that case
    int total;
    if (staged) {
        // thread tid owns frames [lo, hi); coalesced enough for the few KB involved
        const int seg = (n + 255) / 256;
        const int lo = tid * seg < n ? tid * seg : n;
        const int hi = lo + seg < n ? lo + seg : n;
        int sum = 0;
        for (int j = lo; j < hi; ++j) {
            const int c = counts[j];
            soff[j] = c;
            sum += c;
        }
        int incl = sum;
#pragma unroll
        for (int sft = 1; sft < 64; sft <<= 1) {
            const int u = __shfl_up(incl, sft);
            if (lane >= sft) incl += u;
        }
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        int before = 0, all = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            before += q < wave ? wave_tot[q] : 0;
            all += wave_tot[q];
        }
        total = all;
        int run = before + incl - sum;           // exclusive prefix of this thread's frames
        for (int j = lo; j < hi; ++j) {
            const int c = soff[j];
            soff[j] = run;
            if (blockIdx.x == 0) offsets[j] = run;
            run += c;
        }
        if (tid == 255) {
            soff[n] = total;
            if (blockIdx.x == 0) offsets[n] = total;
        }
        __syncthreads();
    } else {
        total = offsets[n];
    }
    const int units = row_bytes / 16;
    for (int j = blockIdx.x * 4 + wave; j < total; j += gridDim.x * 4) {
        int lo = 0, hi = n;                  // offsets[lo] <= j < offsets[hi]
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            const int v = staged ? soff[mid] : offsets[mid];
            if (v <= j) lo = mid; else hi = mid;
        }
        const int first = staged ? soff[lo] : offsets[lo];
        const int src_row = local_idx[(size_t)lo * f + (j - first)];
        if (lane == 0) out_idx[j] = src_row;
        const uint4* src = reinterpret_cast<const uint4*>(feats + (size_t)src_row * row_bytes);
        uint4* dst = reinterpret_cast<uint4*>(out_feats + (size_t)j * row_bytes);
        for (int u0 = lane; u0 < units; u0 += 64 * 8) {          // eight 16-byte loads in flight per lane
            uint4 v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {                        // loads carry no predicate (index clamped)
                const int u = u0 + 64 * k;
                v[k] = load_stream(src + (u < units ? u : units - 1));
            }
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (u0 + 64 * k < units) store_stream(dst + u0 + 64 * k, v[k]);
        }
    }
}

// ---------------------------------------------------------------------------- host side
static int num_compute_units() {
    // asked once per process (devices of one machine are alike); the initialisation of a local static
    // is safe against concurrent first calls
    static const int cached = [] {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
            cus = 256;
        return cus;
    }();
    return cached;
}

int launch_prune_tokens(const TokArgs& a) {
    hipStream_t st = a.stream;
    TokWorkspace ws = carve_tok_workspace(a.workspace, a.n, a.f, a.d, a.dtype);
    const int n_rows = a.n * a.f;
    const int slabs = tok_num_slabs(a.d);
    const size_t esz = a.dtype == SHARPV_F32 ? 4 : 2;
    const bool fused = tok_uses_slab(a.dtype, a.f);

    if (fused) {
        // equal runs of (slab, frame) pairs, about one workgroup per compute unit
        const long long pairs = (long long)slabs * a.n;
        const int wgs = pairs < num_compute_units() ? (int)pairs : num_compute_units();
        const int run_len = (int)(pairs / wgs), run_extra = (int)(pairs % wgs);   // run_len <= n * slabs / 1 fits: n < 2^31
        const dim3 grid(wgs), block(kSlabThreads);
        TimedLaunch tl(kFrameSlab, st);
        switch ((a.f + 15) / 16) {
#define SHARPV_SLAB_CASE(KR)                                                                                     \
    case KR:                                                                                                     \
        hipLaunchKernelGGL(frame_slab_kernel<KR>, grid, block, 0, st, (const bf16_t*)a.feats, a.n, a.f, a.d,     \
                           slabs, run_len, run_extra, ws.aa, ws.am, ws.ab, ws.part_mm);                                      \
        break;
            SHARPV_SLAB_CASE(1) SHARPV_SLAB_CASE(2) SHARPV_SLAB_CASE(3) SHARPV_SLAB_CASE(4) SHARPV_SLAB_CASE(5)
            SHARPV_SLAB_CASE(6) SHARPV_SLAB_CASE(7) SHARPV_SLAB_CASE(8) SHARPV_SLAB_CASE(9) SHARPV_SLAB_CASE(10)
            SHARPV_SLAB_CASE(11) SHARPV_SLAB_CASE(12) SHARPV_SLAB_CASE(13)
#undef SHARPV_SLAB_CASE
            default: return SHARPV_ERR_SHAPE;    // tok_uses_slab admits f <= 208 only
        }
    } else {
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
        TimedLaunch tl(kTokenDots, st);
        if (a.dtype == SHARPV_BF16) launch_token_dots<bf16_t>(a, ws);
        else launch_token_dots<float>(a, ws);
    }
    if (hipGetLastError() != hipSuccess) return SHARPV_ERR_DEVICE;

    {
        TimedLaunch tl(kFrameSelect, st);
        const int tpp = (a.f + 63) / 64 * 64;
        const int parts = 1024 / tpp;            // >= 1 since f <= 1024
        // more frames than compute units: the variant of which two workgroups fit a compute unit
        const bool two_per_cu = a.n > num_compute_units();
#define SHARPV_SELECT_LAUNCH(SB)                                                                                    \
    hipLaunchKernelGGL(frame_select_kernel<SB>, dim3(a.n), dim3(tpp * parts), 0, st,                                \
                       fused ? (const float*)nullptr : (const float*)ws.mean, (const float*)ws.part_mm,             \
                       (const float*)ws.aa, (const float*)ws.am, (const float*)ws.ab, ws.nparts, (size_t)n_rows,    \
                       a.frame_offsets, a.B, a.f, a.d, a.w, a.mode, a.K, a.min_keep, a.measure, tpp, ws.local_idx,  \
                       a.out_counts, a.out_scores, a.out_ratio)
        if (two_per_cu) SHARPV_SELECT_LAUNCH(8);
        else SHARPV_SELECT_LAUNCH(16);
#undef SHARPV_SELECT_LAUNCH
    }
    if (hipGetLastError() != hipSuccess) return SHARPV_ERR_DEVICE;

    const bool self_scan = a.n + 1 <= kOffsetsInLds;
    if (!self_scan) {
        TimedLaunch tl(kCountScan, st);
        hipLaunchKernelGGL(count_scan_kernel, dim3(1), dim3(1024), 0, st, (const int32_t*)a.out_counts, a.n,
                           a.out_offsets);
        if (hipGetLastError() != hipSuccess) return SHARPV_ERR_DEVICE;
    }

    {
        TimedLaunch tl(kTokenGather, st);
        const int want = (n_rows + 3) / 4;
        hipLaunchKernelGGL(token_gather_kernel, dim3(want < 2048 ? want : 2048), dim3(256), 0, st,
                           (const char*)a.feats, (int)(a.d * esz), a.n, a.f,
                           self_scan ? (const int32_t*)a.out_counts : (const int32_t*)nullptr, a.out_offsets,
                           (const int32_t*)ws.local_idx, a.out_idx, (char*)a.out_feats);
    }
    if (hipGetLastError() != hipSuccess) return SHARPV_ERR_DEVICE;
    return SHARPV_OK;
}

}  // namespace sharpv
