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

// Halving tree over the 32 lanes of each half-wavefront.  Every lane of a half ends up with the
// value the written order assigns to leaf 0 (float addition is commutative, so the butterfly
// reproduces p[l] + p[l+s] exactly).
__device__ __forceinline__ float tree32(float v) {
    v = v + __shfl_xor(v, 16);
    v = v + __shfl_xor(v, 8);
    v = v + __shfl_xor(v, 4);
    v = v + __shfl_xor(v, 2);
    v = v + __shfl_xor(v, 1);
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

}  // namespace sharpv
