// Measurement aids of libsharpv (declared in include/sharpv_bench.h), kept apart from the method's
// entry points: per-kernel event timing around the launches of the pruning calls, and a plain
// streaming copy / read that give the device's practical HBM rates.
#include <string.h>

#include <atomic>
#include <mutex>
#include <vector>

#include "../../include/sharpv_bench.h"
#include "sharpv_kernels.hpp"

namespace sharpv {

// ---------------------------------------------------------------------------- event timing
// One process-wide pool of event pairs.  A launch reserves a pair under the lock and keeps its index,
// so host threads that launch at the same time each time their own launch; `generation` changes when
// the pool is rebuilt, which makes a launch that straddles enable / disable drop its record.
namespace {
struct TimingPool {
    std::mutex mutex;
    std::atomic<bool> enabled{false};
    std::vector<hipEvent_t> start, stop;
    std::vector<int> kernel;        // kernel id of each reserved pair
    std::vector<char> closed;       // stop event recorded
    size_t used = 0;
    unsigned generation = 0;
} g_timing;

const char* const kKernelNames[kNumKernels] = {"frame_slab", "frame_mean", "token_dots", "frame_select", "count_scan",
                                               "token_gather", "kv_cosine", "kv_mean", "kv_mask_scan", "kv_gather",
                                               "kv_gather_rope", "stream_copy", "stream_read", "stream_read_slabs",
                                               "stream_gather_rows"};
}  // namespace

long long timing_begin(int kernel, hipStream_t st) {
    TimingPool& t = g_timing;
    if (!t.enabled.load(std::memory_order_acquire)) return -1;      // the common case: no lock taken
    std::lock_guard<std::mutex> lock(t.mutex);
    if (!t.enabled.load(std::memory_order_relaxed) || t.used >= t.start.size()) return -1;
    const size_t slot = t.used++;
    t.kernel[slot] = kernel;
    (void)hipEventRecord(t.start[slot], st);
    return ((long long)t.generation << 32) | (long long)slot;
}

void timing_end(long long ticket, hipStream_t st) {
    if (ticket < 0) return;
    TimingPool& t = g_timing;
    std::lock_guard<std::mutex> lock(t.mutex);
    const size_t slot = (size_t)(ticket & 0xffffffffll);
    if ((unsigned)(ticket >> 32) != t.generation || slot >= t.used) return;      // the pool was rebuilt meanwhile
    (void)hipEventRecord(t.stop[slot], st);
    t.closed[slot] = 1;
}

// with the pool's lock held
static void timing_destroy_locked() {
    TimingPool& t = g_timing;
    t.enabled.store(false, std::memory_order_release);
    for (hipEvent_t e : t.start) (void)hipEventDestroy(e);
    for (hipEvent_t e : t.stop) (void)hipEventDestroy(e);
    t.start.clear();
    t.stop.clear();
    t.kernel.clear();
    t.closed.clear();
    t.used = 0;
    ++t.generation;
}

// ---------------------------------------------------------------------------- measurement aids
__global__ __launch_bounds__(256) void stream_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                          size_t n16) {
    const size_t stride = (size_t)gridDim.x * 256 * 4;
    for (size_t i = (size_t)blockIdx.x * 256 * 4 + threadIdx.x; i < n16; i += stride) {
        uint4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            v[k] = load_stream(src + (i + (size_t)k * 256 < n16 ? i + (size_t)k * 256 : n16 - 1));
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (i + (size_t)k * 256 < n16) store_stream(dst + i + (size_t)k * 256, v[k]);
    }
}

__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ src, size_t n16,
                                                          uint32_t* __restrict__ sink) {
    const size_t stride = (size_t)gridDim.x * 256 * 4;
    uint32_t acc = 0;
    for (size_t i = (size_t)blockIdx.x * 256 * 4 + threadIdx.x; i < n16; i += stride) {
        uint4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            v[k] = load_stream(src + (i + (size_t)k * 256 < n16 ? i + (size_t)k * 256 : i));
#pragma unroll
        for (int k = 0; k < 4; ++k) acc ^= v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
    }
    if (acc == 0x5ca1ab1eu) sink[0] = acc;
}


// The pre-LLM stage's access pattern with the arithmetic taken out: as many workgroups as compute units,
// each walking a run of consecutive (256-column slab, frame) pairs, 512 threads = 16 row groups x 32 lanes,
// every thread reading 16 bytes of rows g, g+16, ... of the frame slab, one frame slab of loads in flight
// while the one before it is consumed.  What this takes is the floor of any kernel that reads the features
// slab by slab, run by run.
constexpr int kPatThreads = 512;
constexpr int kPatRows = 13;        // rows per thread: frames of up to 208 tokens

__global__ __launch_bounds__(kPatThreads) void stream_read_slabs_kernel(const char* __restrict__ feats, int n, int f,
                                                                        int row_bytes, int nslabs, int run_len,
                                                                        int run_extra, uint32_t* __restrict__ sink) {
    const int l = threadIdx.x & 31, g = threadIdx.x >> 5;
    const int units = row_bytes / 16;
    const size_t frame_bytes = (size_t)f * row_bytes;
    uint32_t off[kPatRows];
    uint32_t acc = 0;
    const int w = blockIdx.x;
    long long u = (long long)w * run_len + (w < run_extra ? w : run_extra);
    const long long u_end = u + run_len + (w < run_extra ? 1 : 0);
    while (u < u_end) {
        const int slab = (int)(u / n);
        const int t0 = (int)(u - (long long)slab * n);
        const int t1 = (long long)t0 + (u_end - u) < n ? t0 + (int)(u_end - u) : n;
        const int c = slab * 32 + l;
        const uint32_t chunk_off = (uint32_t)((c < units ? c : units - 1) * 16);
#pragma unroll
        for (int k = 0; k < kPatRows; ++k) {
            const int i = g + 16 * k;
            off[k] = (uint32_t)(i < f ? i : f - 1) * (uint32_t)row_bytes + chunk_off;
        }
        // frames t0 .. t1 (the frame after the run included, as the real kernel reads it for x.x_prev)
        const int last = t1 < n ? t1 : n - 1;
        uint4 a[kPatRows], b[kPatRows];
        const char* base = feats + (size_t)t0 * frame_bytes;
#pragma unroll
        for (int k = 0; k < kPatRows; ++k) a[k] = load_stream(reinterpret_cast<const uint4*>(base + off[k]));
        for (int t = t0; t < last; t += 2) {
            const char* nb = feats + (size_t)(t + 1) * frame_bytes;
#pragma unroll
            for (int k = 0; k < kPatRows; ++k) b[k] = load_stream(reinterpret_cast<const uint4*>(nb + off[k]));
#pragma unroll
            for (int k = 0; k < kPatRows; ++k) acc ^= a[k].x ^ a[k].y ^ a[k].z ^ a[k].w;
            const char* nb2 = feats + (size_t)(t + 2 <= last ? t + 2 : last) * frame_bytes;
#pragma unroll
            for (int k = 0; k < kPatRows; ++k) a[k] = load_stream(reinterpret_cast<const uint4*>(nb2 + off[k]));
#pragma unroll
            for (int k = 0; k < kPatRows; ++k) acc ^= b[k].x ^ b[k].y ^ b[k].z ^ b[k].w;
        }
#pragma unroll
        for (int k = 0; k < kPatRows; ++k) acc ^= a[k].x ^ a[k].y ^ a[k].z ^ a[k].w;
        u += t1 - t0;
    }
    if (acc == 0x5ca1ab1eu) sink[0] = acc;
}

// Indexed row copy: dst row j = src row idx[j], one wavefront per row, 16-byte units, eight in flight per
// lane.  The floor of a compaction whose indices are already known.
__global__ __launch_bounds__(256) void stream_gather_rows_kernel(const char* __restrict__ src, int row_bytes,
                                                                 const int32_t* __restrict__ idx, int n_idx,
                                                                 char* __restrict__ dst) {
    const int lane = threadIdx.x & 63;
    const int units = row_bytes / 16;
    for (int j = blockIdx.x * 4 + (threadIdx.x >> 6); j < n_idx; j += gridDim.x * 4) {
        const uint4* s = reinterpret_cast<const uint4*>(src + (size_t)idx[j] * row_bytes);
        uint4* d = reinterpret_cast<uint4*>(dst + (size_t)j * row_bytes);
        for (int u0 = lane; u0 < units; u0 += 64 * 8) {
            uint4 v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int u = u0 + 64 * k;
                v[k] = load_stream(s + (u < units ? u : units - 1));
            }
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (u0 + 64 * k < units) store_stream(d + u0 + 64 * k, v[k]);
        }
    }
}

static bool aligned16(const void* p) { return ((uintptr_t)p % 16) == 0; }

}  // namespace sharpv

using namespace sharpv;

extern "C" {

int sharpv_stream_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (dst == nullptr || src == nullptr) return SHARPV_ERR_NULL;
    if (bytes == 0 || bytes % 16 != 0 || !aligned16(dst) || !aligned16(src)) return SHARPV_ERR_SHAPE;
    const size_t n16 = bytes / 16;
    const size_t want = (n16 + 1023) / 1024;
    const unsigned grid = (unsigned)(want < 256 * 16 ? want : 256 * 16);
    {
        TimedLaunch tl(kStreamCopy, (hipStream_t)stream);
        hipLaunchKernelGGL(stream_copy_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const uint4*)src,
                           (uint4*)dst, n16);
    }
    return hipGetLastError() == hipSuccess ? SHARPV_OK : SHARPV_ERR_DEVICE;
}

int sharpv_stream_read(const void* src, size_t bytes, uint32_t* sink, void* stream) {
    if (src == nullptr || sink == nullptr) return SHARPV_ERR_NULL;
    if (bytes == 0 || bytes % 16 != 0 || !aligned16(src) || ((uintptr_t)sink % 4) != 0) return SHARPV_ERR_SHAPE;
    const size_t n16 = bytes / 16;
    const size_t want = (n16 + 1023) / 1024;
    const unsigned grid = (unsigned)(want < 256 * 16 ? want : 256 * 16);
    {
        TimedLaunch tl(kStreamRead, (hipStream_t)stream);
        hipLaunchKernelGGL(stream_read_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const uint4*)src, n16,
                           sink);
    }
    return hipGetLastError() == hipSuccess ? SHARPV_OK : SHARPV_ERR_DEVICE;
}

int sharpv_stream_read_slabs(const void* feats, int n_frames, int f, int d, int elem_bytes, uint32_t* sink, void* stream) {
    if (feats == nullptr || sink == nullptr) return SHARPV_ERR_NULL;
    if (n_frames < 1 || f < 1 || f > 16 * kPatRows || d < 8 || (elem_bytes != 2 && elem_bytes != 4) ||
        ((long long)d * elem_bytes) % 16 != 0 || !aligned16(feats) || ((uintptr_t)sink % 4) != 0)
        return SHARPV_ERR_SHAPE;
    const int row_bytes = d * elem_bytes;
    const int nslabs = (row_bytes + 511) / 512;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        return SHARPV_ERR_DEVICE;
    const long long pairs = (long long)nslabs * n_frames;
    const int wgs = pairs < cus ? (int)pairs : cus;
    {
        TimedLaunch tl(kStreamReadSlabs, (hipStream_t)stream);
        hipLaunchKernelGGL(stream_read_slabs_kernel, dim3(wgs), dim3(kPatThreads), 0, (hipStream_t)stream,
                           (const char*)feats, n_frames, f, row_bytes, nslabs, (int)(pairs / wgs), (int)(pairs % wgs), sink);
    }
    return hipGetLastError() == hipSuccess ? SHARPV_OK : SHARPV_ERR_DEVICE;
}

int sharpv_stream_gather_rows(void* dst, const void* src, int row_bytes, const int32_t* idx, int n_idx, void* stream) {
    if (dst == nullptr || src == nullptr || idx == nullptr) return SHARPV_ERR_NULL;
    if (row_bytes < 16 || row_bytes % 16 != 0 || n_idx < 1 || !aligned16(dst) || !aligned16(src) ||
        ((uintptr_t)idx % 4) != 0)
        return SHARPV_ERR_SHAPE;
    const int want = (n_idx + 3) / 4;
    {
        TimedLaunch tl(kStreamGatherRows, (hipStream_t)stream);
        hipLaunchKernelGGL(stream_gather_rows_kernel, dim3(want < 2048 ? want : 2048), dim3(256), 0, (hipStream_t)stream,
                           (const char*)src, row_bytes, idx, n_idx, (char*)dst);
    }
    return hipGetLastError() == hipSuccess ? SHARPV_OK : SHARPV_ERR_DEVICE;
}

int sharpv_timing_enable(int max_launches) {
    TimingPool& t = g_timing;
    std::lock_guard<std::mutex> lock(t.mutex);
    timing_destroy_locked();
    if (max_launches < 1) return SHARPV_ERR_SHAPE;
    t.start.resize((size_t)max_launches);
    t.stop.resize((size_t)max_launches);
    t.kernel.assign((size_t)max_launches, -1);
    t.closed.assign((size_t)max_launches, 0);
    for (int i = 0; i < max_launches; ++i) {
        if (hipEventCreate(&t.start[(size_t)i]) != hipSuccess || hipEventCreate(&t.stop[(size_t)i]) != hipSuccess) {
            t.start.resize((size_t)i);
            t.stop.resize((size_t)i);
            timing_destroy_locked();
            return SHARPV_ERR_DEVICE;
        }
    }
    t.enabled.store(true, std::memory_order_release);
    return SHARPV_OK;
}

int sharpv_timing_disable(void) {
    std::lock_guard<std::mutex> lock(g_timing.mutex);
    timing_destroy_locked();
    return SHARPV_OK;
}

int sharpv_timing_read(const char* kernel_name, int* n_launches, double* total_ms) {
    if (kernel_name == nullptr || n_launches == nullptr || total_ms == nullptr) return SHARPV_ERR_NULL;
    int id = -1;
    for (int k = 0; k < kNumKernels; ++k)
        if (strcmp(kernel_name, kKernelNames[k]) == 0) id = k;
    if (id < 0) return SHARPV_ERR_PARAM;
    TimingPool& t = g_timing;
    std::lock_guard<std::mutex> lock(t.mutex);
    int cnt = 0;
    double tot = 0.0;
    for (size_t i = 0; i < t.used; ++i) {
        if (t.kernel[i] != id || !t.closed[i]) continue;
        if (hipEventSynchronize(t.stop[i]) != hipSuccess) return SHARPV_ERR_DEVICE;
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, t.start[i], t.stop[i]) != hipSuccess) return SHARPV_ERR_DEVICE;
        tot += (double)ms;
        ++cnt;
    }
    *n_launches = cnt;
    *total_ms = tot;
    return SHARPV_OK;
}

}  // extern "C"
