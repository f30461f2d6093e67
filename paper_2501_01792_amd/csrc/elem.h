// The two 16-bit storage formats of activations, weights and K/V: what differs between them in the kernels
// (vector types, the MFMA and dot-product instructions); conversions to and from fp32 are the language's.
// DT is the dtype code of the C ABI (0: fp16, 1: bf16).
#pragma once
#include <hip/hip_runtime.h>

namespace hk {

typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float16v_t __attribute__((ext_vector_type(16)));

template <int DT>
struct Elem;

template <>
struct Elem<0> {
    typedef _Float16 T;
    typedef _Float16 V2 __attribute__((ext_vector_type(2)));
    typedef _Float16 V8 __attribute__((ext_vector_type(8)));
    static __device__ __forceinline__ float4_t mfma_16x16x32(V8 a, V8 b, float4_t c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ float16v_t mfma_32x32x16(V8 a, V8 b, float16v_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ float dot2(V2 a, V2 b, float c) { return __builtin_amdgcn_fdot2(a, b, c, false); }
};

template <>
struct Elem<1> {
    typedef __bf16 T;
    typedef __bf16 V2 __attribute__((ext_vector_type(2)));
    typedef __bf16 V8 __attribute__((ext_vector_type(8)));
    static __device__ __forceinline__ float4_t mfma_16x16x32(V8 a, V8 b, float4_t c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ float16v_t mfma_32x32x16(V8 a, V8 b, float16v_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ float dot2(V2 a, V2 b, float c) { return __builtin_amdgcn_fdot2_f32_bf16(a, b, c, false); }
};

}  // namespace hk
