// Shared device helpers for the gfx950 kernels: bf16 bit handling, wave64
// shuffles, launch-error plumbing.  Written for wave64 CDNA4 only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dllm {

constexpr int kWave = 64;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float floatx4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(16))) float floatx16;

// bf16 is the upper half of a binary32.
__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// Round to nearest even; NaN stays NaN.  Written as a type conversion so that gfx950's
// v_cvt_pk_bf16_f32 does it in one instruction per pair (the integer formulation costs ~10).
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_native;
typedef __attribute__((ext_vector_type(2))) float floatx2_native;
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    const floatx2_native v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_native));
}
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f)
{
    return (uint16_t)(pack_bf16x2(f, 0.0f) & 0xffffu);
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

}  // namespace dllm
