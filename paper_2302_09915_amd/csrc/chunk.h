// 16-byte chunks of a token row as fp32 lanes: unpack / multiply-accumulate / round and pack,
// for the three storage types.  Shared by the combine and by the backward kernels.
#pragma once

#include "internal.h"

namespace tamoe {

template <int DT>
struct Chunk;

template <>
struct Chunk<TAMOE_F32> {
    static constexpr int kElems = 4;
    static __device__ __forceinline__ void fma(float (&acc)[8], float w, vec16 v) {
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = __builtin_fmaf(w, __uint_as_float(v[i]), acc[i]);
    }
    static __device__ __forceinline__ vec16 pack(const float (&acc)[8]) {
        vec16 r;
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = __float_as_uint(acc[i]);
        return r;
    }
};

// fp32 -> bfloat16, round to nearest, ties to even (finite inputs; NaN stays NaN)
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

template <>
struct Chunk<TAMOE_BF16> {
    static constexpr int kElems = 8;
    static __device__ __forceinline__ void fma(float (&acc)[8], float w, vec16 v) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc[2 * i] = __builtin_fmaf(w, __uint_as_float(v[i] << 16), acc[2 * i]);
            acc[2 * i + 1] = __builtin_fmaf(w, __uint_as_float(v[i] & 0xffff0000u), acc[2 * i + 1]);
        }
    }
    static __device__ __forceinline__ vec16 pack(const float (&acc)[8]) {
        vec16 r;
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = f32_to_bf16(acc[2 * i]) | (f32_to_bf16(acc[2 * i + 1]) << 16);
        return r;
    }
};

// IEEE half precision: widening is exact, narrowing rounds to nearest even (the conversion
// instruction under the default rounding mode), overflow goes to infinity.
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

template <>
struct Chunk<TAMOE_F16> {
    static constexpr int kElems = 8;
    static __device__ __forceinline__ void fma(float (&acc)[8], float w, vec16 v) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t u = v[i];  // through a scalar: a bit cast of the vector element itself is miscompiled
            const half2_t h = __builtin_bit_cast(half2_t, u);
            acc[2 * i] = __builtin_fmaf(w, (float)h[0], acc[2 * i]);
            acc[2 * i + 1] = __builtin_fmaf(w, (float)h[1], acc[2 * i + 1]);
        }
    }
    static __device__ __forceinline__ vec16 pack(const float (&acc)[8]) {
        vec16 r;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const half2_t h = {(_Float16)acc[2 * i], (_Float16)acc[2 * i + 1]};
            r[i] = __builtin_bit_cast(uint32_t, h);
        }
        return r;
    }
};

// dot product of the elements of two chunks, accumulated onto acc in element order
template <int DT>
__device__ __forceinline__ float chunk_dot(vec16 a, vec16 b, float acc);

template <>
__device__ __forceinline__ float chunk_dot<TAMOE_F32>(vec16 a, vec16 b, float acc) {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc = __builtin_fmaf(__uint_as_float(a[i]), __uint_as_float(b[i]), acc);
    return acc;
}

template <>
__device__ __forceinline__ float chunk_dot<TAMOE_BF16>(vec16 a, vec16 b, float acc) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        acc = __builtin_fmaf(__uint_as_float(a[i] << 16), __uint_as_float(b[i] << 16), acc);
        acc = __builtin_fmaf(__uint_as_float(a[i] & 0xffff0000u), __uint_as_float(b[i] & 0xffff0000u), acc);
    }
    return acc;
}

template <>
__device__ __forceinline__ float chunk_dot<TAMOE_F16>(vec16 a, vec16 b, float acc) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t ua = a[i], ub = b[i];
        const half2_t x = __builtin_bit_cast(half2_t, ua), y = __builtin_bit_cast(half2_t, ub);
        acc = __builtin_fmaf((float)x[0], (float)y[0], acc);
        acc = __builtin_fmaf((float)x[1], (float)y[1], acc);
    }
    return acc;
}

}  // namespace tamoe
