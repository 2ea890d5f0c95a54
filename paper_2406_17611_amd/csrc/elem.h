// Storage element types of activations and gradients: fp32, or bf16 with fp32 arithmetic. Loads convert to
// float, stores round to nearest even.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

struct bf16_t {
    uint16_t bits;
};

__device__ __forceinline__ float bf16_to_float(uint16_t b) { return __uint_as_float(uint32_t(b) << 16); }

// Round to nearest even (the hardware conversion of gfx950); NaN stays NaN.
__device__ __forceinline__ uint16_t float_to_bf16(float f) { return __builtin_bit_cast(uint16_t, static_cast<__bf16>(f)); }

template <typename T>
struct Elem;

template <>
struct Elem<float> {
    static __device__ __forceinline__ float load(const float* p) { return *p; }
    static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
    static __device__ __forceinline__ float2 load2(const float* p) { return *reinterpret_cast<const float2*>(p); }
    static __device__ __forceinline__ float4 load4(const float* p) { return *reinterpret_cast<const float4*>(p); }
    static __device__ __forceinline__ void store2(float* p, float2 v) { *reinterpret_cast<float2*>(p) = v; }
    static __device__ __forceinline__ void store4(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
};

template <>
struct Elem<bf16_t> {
    static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_float(p->bits); }
    static __device__ __forceinline__ void store(bf16_t* p, float v) { p->bits = float_to_bf16(v); }
    static __device__ __forceinline__ float2 load2(const bf16_t* p) {
        const uint32_t u = *reinterpret_cast<const uint32_t*>(p);
        return make_float2(__uint_as_float(u << 16), __uint_as_float(u & 0xFFFF0000u));
    }
    static __device__ __forceinline__ float4 load4(const bf16_t* p) {
        const uint2 u = *reinterpret_cast<const uint2*>(p);
        return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xFFFF0000u), __uint_as_float(u.y << 16),
                           __uint_as_float(u.y & 0xFFFF0000u));
    }
    static __device__ __forceinline__ void store2(bf16_t* p, float2 v) {
        *reinterpret_cast<uint32_t*>(p) = uint32_t(float_to_bf16(v.x)) | (uint32_t(float_to_bf16(v.y)) << 16);
    }
    static __device__ __forceinline__ void store4(bf16_t* p, float4 v) {
        uint2 u;
        u.x = uint32_t(float_to_bf16(v.x)) | (uint32_t(float_to_bf16(v.y)) << 16);
        u.y = uint32_t(float_to_bf16(v.z)) | (uint32_t(float_to_bf16(v.w)) << 16);
        *reinterpret_cast<uint2*>(p) = u;
    }
};

// Loads / stores of N = 1, 2 or 4 consecutive elements as a float vector type.
template <int N>
struct FloatVec;
template <>
struct FloatVec<1> {
    using type = float;
};
template <>
struct FloatVec<2> {
    using type = float2;
};
template <>
struct FloatVec<4> {
    using type = float4;
};

template <typename T, int N>
__device__ __forceinline__ typename FloatVec<N>::type load_vec(const T* p) {
    if constexpr (N == 4)
        return Elem<T>::load4(p);
    else if constexpr (N == 2)
        return Elem<T>::load2(p);
    else
        return Elem<T>::load(p);
}

template <typename T, int N>
__device__ __forceinline__ void store_vec(T* p, typename FloatVec<N>::type v) {
    if constexpr (N == 4)
        Elem<T>::store4(p, v);
    else if constexpr (N == 2)
        Elem<T>::store2(p, v);
    else
        Elem<T>::store(p, v);
}
