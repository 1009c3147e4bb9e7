// Device-side helpers shared by the HIP kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tweo {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

__device__ __forceinline__ float bits_to_f32(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t f32_to_bits(float f) { return __builtin_bit_cast(uint32_t, f); }

// A dword holds two bf16; widening is a shift / mask.
__device__ __forceinline__ float bf16lo_to_f32(uint32_t d) { return bits_to_f32(d << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t d) { return bits_to_f32(d & 0xFFFF0000u); }

// Two fp32 -> packed bf16 pair (round to nearest even, v_cvt_pk_bf16_f32); lo in bits 15:0.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    v2f v = {lo, hi};
    bf16x2 b = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(uint32_t, b);
}

// Per-tensor scale into an 8-bit float range (Sec. 4.3; E4M3: +-448 from Sec. 1, E5M2: +-57344):
// range/amax as one IEEE fp32 division; amax of 0 / Inf / NaN -> 1; overflow -> FLT_MAX.
__device__ __forceinline__ float scale_from_amax_range(float amax, float range)
{
    float s = 1.0f;
    if (amax > 0.0f && amax < __builtin_inff()) {
        s = range / amax;
        if (s == __builtin_inff())
            s = 3.402823466e+38f;
    }
    return s;
}

__device__ __forceinline__ float scale_from_amax(float amax) { return scale_from_amax_range(amax, 448.0f); }

// Eq. 4 rounding to INT8: clamp(rne(v * inv_step), +-127), NaN -> 0; the low byte of the result
__device__ __forceinline__ uint32_t round_to_i8(float v, float inv_step)
{
    const float prod = v * inv_step;
    float r = __builtin_rintf(prod);  // v_rndne_f32: ties to even
    r = __builtin_amdgcn_fmed3f(r, -127.0f, 127.0f);
    r = (prod != prod) ? 0.0f : r;
    return (uint32_t)(int)r & 0xFFu;
}

template <typename T>
__device__ __forceinline__ T wave_reduce_sum(T v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
        v += __shfl_xor(v, off, kWave);
    return v;
}

__device__ __forceinline__ uint32_t wave_reduce_max_u32(uint32_t v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        uint32_t o = (uint32_t)__shfl_xor((int)v, off, kWave);
        v = o > v ? o : v;
    }
    return v;
}

}  // namespace tweo
