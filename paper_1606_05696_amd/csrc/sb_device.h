// Device helpers shared by the kernels: element types and conversions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// bf16 element: the upper 16 bits of an fp32 number.
struct sb_bf16 { uint16_t bits; };

__device__ __forceinline__ float sb_bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// fp32 -> bf16, round to nearest, ties to even; NaN stays NaN (quiet).
__device__ __forceinline__ uint16_t sb_f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <typename T, typename Acc> __device__ __forceinline__ Acc sb_load(const T *p) { return (Acc)*p; }
template <> __device__ __forceinline__ float sb_load<sb_bf16, float>(const sb_bf16 *p) { return sb_bf16_to_f32(p->bits); }

template <typename T, typename Acc> __device__ __forceinline__ void sb_store(T *p, Acc v) { *p = (T)v; }
template <> __device__ __forceinline__ void sb_store<sb_bf16, float>(sb_bf16 *p, float v) { p->bits = sb_f32_to_bf16(v); }
