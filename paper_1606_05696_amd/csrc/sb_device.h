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

// 16 bytes per lane from global memory straight into LDS (no staging registers, no LDS store instruction):
// lane l of the wave lands at lds_addr + 16 l.  lds_addr and base are wave-uniform; voff is the lane's byte
// offset from base (unsigned 32 bit).  The compiler does not see the LDS write behind this statement: the
// code that reads the data waits for it itself (dma_wait) before the barrier that publishes it.  M0 is not
// allocated by the compiler and nothing else in these kernels uses it.
__device__ __forceinline__ void dma16(unsigned lds_addr, const void *base, unsigned voff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" :: "s"(lds_addr), "v"(voff), "s"(base) : "memory");
}
// wait until at most N vector-memory operations of this wave are outstanding (they complete in order)
template <int N>
__device__ __forceinline__ void dma_wait()
{
    static_assert(N >= 0 && N < 64, "6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));      // expcnt and lgkmcnt fields: no wait
}
