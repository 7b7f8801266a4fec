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

// Sums N = 2^K values per lane (N = 4, 8 or 16) over the 64 lanes: every step folds the wavefront in
// half and halves the number of values a lane carries (the lanes whose bit `off` is clear keep the
// first half of the values).  On return v[0] of lane l holds the total of value l >> (6 - K).
// The halves 32 and 16 lanes apart change places with the lane-swap instructions (one swap and one
// add per pair of values), the nearer ones with DPP moves (a row rotated by 8, a mirrored half row,
// quads permuted): no step goes through LDS.
template <int N>
__device__ __forceinline__ void wave_fold(float (&v)[N])
{
    static_assert(N == 4 || N == 8 || N == 16, "4, 8 or 16 values");
    const int lane = threadIdx.x & 63;
    typedef unsigned uint2_t __attribute__((ext_vector_type(2)));
    int m = N;
    // 32 lanes apart: after the swap the first register holds [first.low, second.low], the second [first.high, second.high]
#pragma unroll
    for (int i = 0; i < N / 2; ++i) {
        const uint2_t sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(v[i]), __float_as_uint(v[i + N / 2]), false, false);
        v[i] = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    }
    m = N / 2;
    // 16 lanes apart: odd rows of the first register change places with even rows of the second
#pragma unroll
    for (int i = 0; i < N / 4; ++i) {
        const uint2_t sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(v[i]), __float_as_uint(v[i + N / 4]), false, false);
        v[i] = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    }
    m = N / 4;
    auto dpp = [](float x, auto ctrl) {
        return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, x), decltype(ctrl)::value, 0xF, 0xF, true));
    };
    struct Ror8 { enum { value = 0x128 }; };        // row rotated right by 8: lane ^ 8
    struct HalfMirror { enum { value = 0x141 }; };  // lanes of every 8 reversed: pairs 0..3 with 7..4
    struct Xor2 { enum { value = 0x4E }; };         // quad_perm [2, 3, 0, 1]
    struct Xor1 { enum { value = 0xB1 }; };         // quad_perm [1, 0, 3, 2]
    if constexpr (N >= 8) {  // 8 lanes apart
        const bool upper = (lane & 8) != 0;
#pragma unroll
        for (int i = 0; i < N / 8; ++i) {
            const float lo = v[i], hi = v[i + N / 8];
            const float give = upper ? lo : hi, keep = upper ? hi : lo;
            v[i] = keep + dpp(give, Ror8{});
        }
    } else {
        v[0] += dpp(v[0], Ror8{});
    }
    if constexpr (N >= 16) {  // 4 lanes apart
        const bool upper = (lane & 4) != 0;
        const float lo = v[0], hi = v[1];
        const float give = upper ? lo : hi, keep = upper ? hi : lo;
        v[0] = keep + dpp(give, HalfMirror{});
    } else {
        v[0] += dpp(v[0], HalfMirror{});
    }
    v[0] += dpp(v[0], Xor2{});
    v[0] += dpp(v[0], Xor1{});
    (void)m;
}

}  // namespace lora
