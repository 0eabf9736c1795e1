// Device helpers shared by the kernels: element types and conversions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// bf16 element: the upper 16 bits of an fp32 number.
struct sb_bf16 { uint16_t bits; };

__device__ __forceinline__ float sb_bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// fp32 -> bf16, round to nearest, ties to even; NaN stays NaN.  gfx950 converts in hardware
// (v_cvt_pk_bf16_f32), which is what the cast compiles to.
__device__ __forceinline__ uint16_t sb_f32_to_bf16(float f)
{
    return __builtin_bit_cast(uint16_t, (__bf16)f);
}

template <typename T, typename Acc> __device__ __forceinline__ Acc sb_load(const T *p) { return (Acc)*p; }
template <> __device__ __forceinline__ float sb_load<sb_bf16, float>(const sb_bf16 *p) { return sb_bf16_to_f32(p->bits); }

template <typename T, typename Acc> __device__ __forceinline__ void sb_store(T *p, Acc v) { *p = (T)v; }
template <> __device__ __forceinline__ void sb_store<sb_bf16, float>(sb_bf16 *p, float v) { p->bits = sb_f32_to_bf16(v); }
