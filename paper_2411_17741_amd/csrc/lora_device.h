// Device-side helpers for the gfx950 kernels: 8-element chunks of fp32 / bf16, conversions,
// wavefront reduction.
#pragma once

#include "lora_internal.h"

namespace lora {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// 8 consecutive elements: one 16-byte vector of bf16, two of fp32.
template <typename E> struct Chunk;
template <> struct __attribute__((aligned(16))) Chunk<__bf16> { uint4 v; };
template <> struct __attribute__((aligned(16))) Chunk<float> { float4 lo, hi; };

template <typename E> __device__ __forceinline__ Chunk<E> load_chunk(const E *p)
{
    return *reinterpret_cast<const Chunk<E> *>(p);
}
template <typename E> __device__ __forceinline__ void store_chunk(E *p, const Chunk<E> &c)
{
    *reinterpret_cast<Chunk<E> *>(p) = c;
}
template <typename E> __device__ __forceinline__ Chunk<E> zero_chunk();
template <> __device__ __forceinline__ Chunk<__bf16> zero_chunk<__bf16>()
{
    Chunk<__bf16> c;
    c.v = make_uint4(0, 0, 0, 0);
    return c;
}
template <> __device__ __forceinline__ Chunk<float> zero_chunk<float>()
{
    Chunk<float> c;
    c.lo = make_float4(0, 0, 0, 0);
    c.hi = make_float4(0, 0, 0, 0);
    return c;
}

// bf16 pair packed in a 32-bit word: element 0 in the low half
__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ void unpack_chunk(const Chunk<__bf16> &c, float (&f)[8])
{
    f[0] = bf_lo(c.v.x); f[1] = bf_hi(c.v.x);
    f[2] = bf_lo(c.v.y); f[3] = bf_hi(c.v.y);
    f[4] = bf_lo(c.v.z); f[5] = bf_hi(c.v.z);
    f[6] = bf_lo(c.v.w); f[7] = bf_hi(c.v.w);
}
__device__ __forceinline__ void unpack_chunk(const Chunk<float> &c, float (&f)[8])
{
    f[0] = c.lo.x; f[1] = c.lo.y; f[2] = c.lo.z; f[3] = c.lo.w;
    f[4] = c.hi.x; f[5] = c.hi.y; f[6] = c.hi.z; f[7] = c.hi.w;
}

template <typename E> __device__ __forceinline__ float dot_chunk(const Chunk<E> &a, const Chunk<E> &b)
{
    float fa[8], fb[8];
    unpack_chunk(a, fa);
    unpack_chunk(b, fb);
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += fa[i] * fb[i];
    return s;
}

// acc + dot(a, b) over the 8 elements; bf16 pairs go through the packed dot instruction
// (products are exact in fp32, accumulation is fp32)
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float dot_chunk_acc(float acc, const Chunk<__bf16> &a, const Chunk<__bf16> &b)
{
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.v.x), __builtin_bit_cast(bf16x2, b.v.x), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.v.y), __builtin_bit_cast(bf16x2, b.v.y), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.v.z), __builtin_bit_cast(bf16x2, b.v.z), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.v.w), __builtin_bit_cast(bf16x2, b.v.w), acc, false);
    return acc;
}
__device__ __forceinline__ float dot_chunk_acc(float acc, const Chunk<float> &a, const Chunk<float> &b)
{
    return acc + dot_chunk(a, b);
}

__device__ __forceinline__ float to_float(float v) { return v; }
__device__ __forceinline__ float to_float(__bf16 v) { return (float)v; }
template <typename E> __device__ __forceinline__ E from_float(float v);
template <> __device__ __forceinline__ float from_float<float>(float v) { return v; }
template <> __device__ __forceinline__ __bf16 from_float<__bf16>(float v) { return (__bf16)v; }  // round to nearest even

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Sums N = 2^K values per lane over the 64 lanes with N - 1 + (6 - K) shuffles instead of 6 N:
// every step folds the wavefront in half and halves the number of values a lane carries (the
// lower half of the lanes keeps the first half of the values).  On return v[0] of lane l holds
// the total of value l >> (6 - K).
template <int N>
__device__ __forceinline__ void wave_sum_fold(float (&v)[N])
{
    static_assert(N == 1 || N == 2 || N == 4 || N == 8 || N == 16, "power of two up to 16");
    const int lane = threadIdx.x & 63;
    auto from = [&](float x, int off) {
        return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((lane ^ off) << 2, __builtin_bit_cast(int, x)));
    };
    int off = 32;
#pragma unroll
    for (int m = N; m > 1; m >>= 1, off >>= 1) {
        const bool upper = (lane & off) != 0;
#pragma unroll
        for (int i = 0; i < m / 2; ++i) {
            const float lo = v[i], hi = v[i + m / 2];  // named, so that the selects stay selects of values
            const float give = upper ? lo : hi;
            const float keep = upper ? hi : lo;
            v[i] = keep + from(give, off);
        }
    }
    for (; off > 0; off >>= 1) v[0] += from(v[0], off);
}

}  // namespace lora
