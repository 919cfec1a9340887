// Device-side building blocks shared by the SharpV kernels (gfx950, wave64).
//
// All inner products over the feature dimension follow one fixed order so that results repeat
// bit for bit whatever the launch geometry:
//   - the row is cut into blocks of 256 elements; a block is 32 chunks of 8 consecutive elements;
//   - a chunk is folded by an 8-step fused multiply-add chain starting from +0;
//   - the 32 chunk values of a block are reduced by a halving tree (strides 16, 8, 4, 2, 1);
//   - block values are added to the running total in ascending block order.
// A half-wavefront (32 lanes) owns one block: lane l holds chunk l.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sharpv {

constexpr int kChunk = 8;            // elements per chunk
constexpr int kBlockChunks = 32;     // chunks per block
constexpr int kBlockElems = kChunk * kBlockChunks;   // 256

struct bf16_t { uint16_t bits; };

// Streaming accesses: data that is touched once and should not displace anything in the caches.
__device__ __forceinline__ uint4 load_stream(const uint4* p) {
    uint4 r;
    r.x = __builtin_nontemporal_load(&p->x);
    r.y = __builtin_nontemporal_load(&p->y);
    r.z = __builtin_nontemporal_load(&p->z);
    r.w = __builtin_nontemporal_load(&p->w);
    return r;
}
__device__ __forceinline__ void store_stream(uint4* p, const uint4& v) {
    __builtin_nontemporal_store(v.x, &p->x);
    __builtin_nontemporal_store(v.y, &p->y);
    __builtin_nontemporal_store(v.z, &p->z);
    __builtin_nontemporal_store(v.w, &p->w);
}

// ---------------------------------------------------------------------------- raw chunk loads
template <typename T> struct RawChunk;
template <> struct RawChunk<bf16_t> { uint4 q; };
template <> struct RawChunk<float> { float4 a, b; };

template <typename T> __device__ __forceinline__ RawChunk<T> load_raw(const T* p);

template <> __device__ __forceinline__ RawChunk<bf16_t> load_raw<bf16_t>(const bf16_t* p) {
    RawChunk<bf16_t> r;
    r.q = *reinterpret_cast<const uint4*>(p);
    return r;
}
template <> __device__ __forceinline__ RawChunk<float> load_raw<float>(const float* p) {
    RawChunk<float> r;
    r.a = reinterpret_cast<const float4*>(p)[0];
    r.b = reinterpret_cast<const float4*>(p)[1];
    return r;
}

// The same loads marked as streaming (non-temporal).
template <typename T> __device__ __forceinline__ RawChunk<T> load_raw_stream(const T* p);
template <> __device__ __forceinline__ RawChunk<bf16_t> load_raw_stream<bf16_t>(const bf16_t* p) {
    RawChunk<bf16_t> r;
    r.q = load_stream(reinterpret_cast<const uint4*>(p));
    return r;
}
template <> __device__ __forceinline__ RawChunk<float> load_raw_stream<float>(const float* p) {
    RawChunk<float> r;
    const uint4 a = load_stream(reinterpret_cast<const uint4*>(p));
    const uint4 b = load_stream(reinterpret_cast<const uint4*>(p) + 1);
    r.a = make_float4(__uint_as_float(a.x), __uint_as_float(a.y), __uint_as_float(a.z), __uint_as_float(a.w));
    r.b = make_float4(__uint_as_float(b.x), __uint_as_float(b.y), __uint_as_float(b.z), __uint_as_float(b.w));
    return r;
}

template <typename T> __device__ __forceinline__ RawChunk<T> zero_raw();
template <> __device__ __forceinline__ RawChunk<bf16_t> zero_raw<bf16_t>() {
    RawChunk<bf16_t> r;
    r.q = make_uint4(0u, 0u, 0u, 0u);
    return r;
}
template <> __device__ __forceinline__ RawChunk<float> zero_raw<float>() {
    RawChunk<float> r;
    r.a = make_float4(0.f, 0.f, 0.f, 0.f);
    r.b = r.a;
    return r;
}

// bf16 -> float32 is exact: the 16 bits become the high half of the float.
__device__ __forceinline__ void unpack(const RawChunk<bf16_t>& r, float (&v)[8]) {
    v[0] = __uint_as_float(r.q.x << 16); v[1] = __uint_as_float(r.q.x & 0xffff0000u);
    v[2] = __uint_as_float(r.q.y << 16); v[3] = __uint_as_float(r.q.y & 0xffff0000u);
    v[4] = __uint_as_float(r.q.z << 16); v[5] = __uint_as_float(r.q.z & 0xffff0000u);
    v[6] = __uint_as_float(r.q.w << 16); v[7] = __uint_as_float(r.q.w & 0xffff0000u);
}
__device__ __forceinline__ void unpack(const RawChunk<float>& r, float (&v)[8]) {
    v[0] = r.a.x; v[1] = r.a.y; v[2] = r.a.z; v[3] = r.a.w;
    v[4] = r.b.x; v[5] = r.b.y; v[6] = r.b.z; v[7] = r.b.w;
}

// 8-step fused chain of one chunk, starting from +0.
__device__ __forceinline__ float chain8(const float (&x)[8], const float (&y)[8]) {
    float c = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j) c = __builtin_fmaf(x[j], y[j], c);
    return c;
}

// Lane l of a 16-lane row receives the value of lane (l - n) mod 16 of the same row (DPP row_ror:
// values move towards higher lane numbers).
template <int N> __device__ __forceinline__ float row_rotate(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x120 + N, 0xf, 0xf, false));
}

// Strides 8, 4, 2, 1 of the halving tree inside every 16-lane row.  After the stride-8 step the
// row holds each partial twice (lanes l and l^8), after stride 4 four times, and so on, so a
// rotation by s delivers the partner of stride s whichever way it turns.
__device__ __forceinline__ float tree16_rows(float v) {
    v = v + row_rotate<8>(v);
    v = v + row_rotate<4>(v);
    v = v + row_rotate<2>(v);
    v = v + row_rotate<1>(v);
    return v;
}

// Halving tree over the 32 lanes of each half-wavefront (strides 16, 8, 4, 2, 1).  Every lane of
// a half ends up with the value the written order assigns to leaf 0 (float addition is
// commutative, so the butterfly reproduces p[l] + p[l+s] exactly).  The stride-16 step exchanges
// the two 16-lane rows of a half with v_permlane16_swap.
__device__ __forceinline__ float tree32(float v) {
    const unsigned u = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    return tree16_rows(__uint_as_float(r[0]) + __uint_as_float(r[1]));
}

// Two trees for the price of one: v_permlane16_swap exchanges the odd 16-lane rows of its first
// operand with the even rows of its second, giving {a.r0, b.r0, a.r2, b.r2} and {a.r1, b.r1, a.r3,
// b.r3}; their sum carries a's stride-16 sums in rows 0 and 2 and b's in rows 1 and 3.  Result:
// lanes 0-15 / 32-47 hold TREE32 of `a` (lower / upper half-wavefront), lanes 16-31 / 48-63 hold
// TREE32 of `b`.
__device__ __forceinline__ float tree32_pair(float a, float b) {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    return tree16_rows(__uint_as_float(r[0]) + __uint_as_float(r[1]));
}

// Four trees at a time.  The stride-16 step runs as in tree32_pair for (a, b) and for (c, d); at
// stride 8 lanes 0-7 of every 16-lane row go on with the first pair and lanes 8-15 with the second
// (each takes its own value and receives its stride-8 partner's by a rotation of the other
// selection), and strides 4, 2, 1 are shared.  A rotation by s < 8 hands lane l the value of lane
// l - s, so inside a group of 8 only lanes >= 4, then >= 6, then lane 7 keep receiving partners of
// their own tree: lanes 7 / 15 / 23 / 31 of a half-wavefront end with TREE32 of a / c / b / d (the
// same additions as the halving tree, operands swapped), the other lanes with mixtures.
__device__ __forceinline__ float tree32_quad(float a, float b, float c, float d) {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    const auto s = __builtin_amdgcn_permlane16_swap(__float_as_uint(c), __float_as_uint(d), false, false);
    const float x = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    const float y = __uint_as_float(s[0]) + __uint_as_float(s[1]);
    const bool upper = (threadIdx.x & 8) != 0;
    const float own = upper ? y : x;
    const float other = upper ? x : y;
    float v = own + row_rotate<8>(other);
    v = v + row_rotate<4>(v);
    v = v + row_rotate<2>(v);
    v = v + row_rotate<1>(v);
    return v;
}

__device__ __forceinline__ float lane_value(float v, int lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

// Adds the block values held by the two halves of a wavefront (even block in lanes 0-31, odd
// block in lanes 32-63) to the running total, in ascending block order.
__device__ __forceinline__ float add_blocks(float acc, float tree_value, bool odd_block_exists) {
    acc = acc + lane_value(tree_value, 0);
    if (odd_block_exists) acc = acc + lane_value(tree_value, 32);
    return acc;
}

// cos(theta) from the three inner products; a zero (or underflowed) norm product gives 0.
__device__ __forceinline__ float cos_from_dots(float xy, float xx, float yy) {
    // sqrtf and "/" are the correctly rounded ones (the library is built with
    // -fhip-fp32-correctly-rounded-divide-sqrt and -ffp-contract=off).
    const float den = __builtin_sqrtf(xx * yy);
    if (!(den > 0.0f)) return 0.0f;
    float c = xy / den;
    c = c > 1.0f ? 1.0f : c;
    c = c < -1.0f ? -1.0f : c;
    return c;
}

// Eq.1 (second form): sqrt(2 - 2 cos).
__device__ __forceinline__ float dissim_from_dots(float xy, float xx, float yy) {
    const float q = __builtin_fmaf(-2.0f, cos_from_dots(xy, xx, yy), 2.0f);
    return __builtin_sqrtf(fmaxf(q, 0.0f));
}

// S and T of Sec. 3.1 from the three inner products: Eq.1, or (measure 1) the rescaled cosine 1 - cos
// that the same section allows together with a fixed threshold.
__device__ __forceinline__ float measure_from_dots(int measure, float xy, float xx, float yy) {
    return measure == 0 ? dissim_from_dots(xy, xx, yy) : 1.0f - cos_from_dots(xy, xx, yy);
}

// Inclusive integer prefix sum over a 1024-thread workgroup: shuffle scan inside each wavefront,
// the 16 wavefront totals through LDS.  (Integers: any order gives the same sums.)
__device__ __forceinline__ int block_inclusive_scan_1024(int v, int* wave_tot /* LDS [16] */) {
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
        const int u = __shfl_up(v, s);
        if (lane >= s) v += u;
    }
    if (lane == 63) wave_tot[wave] = v;
    __syncthreads();
    int before = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) before += w < wave ? wave_tot[w] : 0;
    return v + before;
}

}  // namespace sharpv
