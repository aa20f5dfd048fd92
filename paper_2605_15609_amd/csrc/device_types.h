// Storage types and conversions used by the device code.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// bf16_t is declared in psd_internal.h as a 2-byte struct holding the raw bits.

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// fp32 -> bf16, round to nearest even: the hardware conversion of gfx950 (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }

__device__ __forceinline__ float to_float(float v) { return v; }
__device__ __forceinline__ float to_float(bf16_t v) { return bf16_bits_to_float(v.bits); }

template <typename T>
__device__ __forceinline__ T from_float(float f);
template <>
__device__ __forceinline__ float from_float<float>(float f) {
    return f;
}
template <>
__device__ __forceinline__ bf16_t from_float<bf16_t>(float f) {
    bf16_t r;
    r.bits = float_to_bf16_bits(f);
    return r;
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    const bf16x2_t v = {(__bf16)lo, (__bf16)hi};   // one instruction for the pair
    return __builtin_bit_cast(uint32_t, v);
}
