// Storage types of activations: fp32, or bf16 (fp32 arithmetic everywhere, bf16 only in memory and as
// MFMA operands).  Kernels are templates on the storage type T; Act<T> moves four consecutive
// channels between memory and an f32x4.
#pragma once
#include "kernels.h"

typedef uint16_t bf16_t;
typedef short s16x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float((uint32_t)h << 16); }

// round to nearest even; NaN stays a quiet NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

template <typename T>
struct Act;

template <>
struct Act<float> {
    typedef f32x4 raw4;  // four channels as stored
    static __device__ __forceinline__ raw4 zero() { return f32x4{0.f, 0.f, 0.f, 0.f}; }
    static __device__ __forceinline__ raw4 load_raw(const float* p) { return *reinterpret_cast<const f32x4*>(p); }
    static __device__ __forceinline__ f32x4 load4(const float* p) { return *reinterpret_cast<const f32x4*>(p); }
    static __device__ __forceinline__ void store4(float* p, f32x4 v) { *reinterpret_cast<f32x4*>(p) = v; }
    static __device__ __forceinline__ f32x4 widen(raw4 r) { return r; }
    static __device__ __forceinline__ f32x4 rounded(f32x4 v) { return v; }  // value as it will read back from memory
};

template <>
struct Act<bf16_t> {
    typedef uint2 raw4;
    static __device__ __forceinline__ raw4 zero() { return make_uint2(0u, 0u); }
    static __device__ __forceinline__ raw4 load_raw(const bf16_t* p) { return *reinterpret_cast<const uint2*>(p); }
    static __device__ __forceinline__ f32x4 widen(raw4 r) {
        return f32x4{__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xffff0000u), __uint_as_float(r.y << 16),
                     __uint_as_float(r.y & 0xffff0000u)};
    }
    static __device__ __forceinline__ f32x4 load4(const bf16_t* p) { return widen(load_raw(p)); }
    // round to nearest even by the hardware's packed conversion (the same values as f32_to_bf16)
    static __device__ __forceinline__ raw4 narrow(f32x4 v) {
        typedef __bf16 bf16x2_hw __attribute__((ext_vector_type(2)));
        typedef float f32x2_hw __attribute__((ext_vector_type(2)));
        return make_uint2(__builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2_hw){v[0], v[1]}, bf16x2_hw)),
                          __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2_hw){v[2], v[3]}, bf16x2_hw)));
    }
    static __device__ __forceinline__ void store4(bf16_t* p, f32x4 v) { *reinterpret_cast<uint2*>(p) = narrow(v); }
    static __device__ __forceinline__ f32x4 rounded(f32x4 v) { return widen(narrow(v)); }
};

// Calls `expr` with T bound to the storage type named by `act` (ACT_F32 / ACT_BF16).
#define ACT_DISPATCH(act, ...)            \
    do {                                  \
        if ((act) == ACT_BF16) {          \
            typedef bf16_t T;             \
            __VA_ARGS__;                  \
        } else {                          \
            typedef float T;              \
            __VA_ARGS__;                  \
        }                                 \
    } while (0)
