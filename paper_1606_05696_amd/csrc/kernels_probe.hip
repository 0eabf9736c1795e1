// Peak-rate probe: a kernel that does nothing but issue MFMAs of the type a StridedBatchedGemm of
// the given element type uses (four independent accumulators per wave, two waves per SIMD), so
// that a benchmark can price its kernels against what the matrix cores of THIS device deliver
// at its sustained clock, next to the published peak.
#include "sb_internal.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef double f64x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int PROBE_BLOCKS = 1024, PROBE_THREADS = 256;      // 4 waves per SIMD on 256 compute units
constexpr int UNROLL = 16;                                   // rounds per loop trip: the loop's own register traffic stays small

template <int DT>
__global__ __launch_bounds__(PROBE_THREADS) void probe_kernel(float *out, float x, int iterations)
{
    float s = 0.f;
    if (DT == SB_F32) {
        f32x16 c[4] = {};
        const float a = x + threadIdx.x, b = x;
        for (int i = 0; i < iterations; i += UNROLL)
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
#pragma unroll
                for (int j = 0; j < 4; ++j) c[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c[j], 0, 0, 0);
        for (int j = 0; j < 4; ++j) s += c[j][0];
    } else if (DT == SB_F64) {
        f64x4 c[4] = {};
        const double a = x + threadIdx.x, b = x;
        for (int i = 0; i < iterations; i += UNROLL)
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
#pragma unroll
                for (int j = 0; j < 4; ++j) c[j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c[j], 0, 0, 0);
        for (int j = 0; j < 4; ++j) s += (float)c[j][0];
    } else {
        f32x16 c[4] = {};
        bf16x8 a, b;
        for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(x + e); b[e] = (__bf16)x; }
        for (int i = 0; i < iterations; i += UNROLL)
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
#pragma unroll
                for (int j = 0; j < 4; ++j) c[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[j], 0, 0, 0);
        for (int j = 0; j < 4; ++j) s += c[j][0];
    }
    out[(size_t)blockIdx.x * PROBE_THREADS + threadIdx.x] = s;
}

}  // namespace

extern "C" int sb_probe_mfma(sb_dtype dt, int iterations, void *scratch, int64_t scratch_bytes, void *stream, double *flops)
{
    if ((int)dt < SB_F64 || (int)dt > SB_BF16) return -1;
    if (iterations < UNROLL || iterations % UNROLL) return -2;
    if (!scratch) return -3;
    if (scratch_bytes < (int64_t)PROBE_BLOCKS * PROBE_THREADS * 4) return -4;
    if (!flops) return -6;
    hipStream_t st = (hipStream_t)stream;
    const int PB = PROBE_BLOCKS;
    // flops of one MFMA: 2 * M * N * K of the instruction
    const double per_mfma = dt == SB_F32 ? 2.0 * 32 * 32 * 2 : (dt == SB_F64 ? 2.0 * 16 * 16 * 4 : 2.0 * 32 * 32 * 16);
    if (dt == SB_F32)      probe_kernel<SB_F32><<<PB, PROBE_THREADS, 0, st>>>((float *)scratch, 1.0f, iterations);
    else if (dt == SB_F64) probe_kernel<SB_F64><<<PB, PROBE_THREADS, 0, st>>>((float *)scratch, 1.0f, iterations);
    else                   probe_kernel<SB_BF16><<<PB, PROBE_THREADS, 0, st>>>((float *)scratch, 1.0f, iterations);
    *flops = per_mfma * 4.0 * iterations * (double)(PB * (PROBE_THREADS / 64));
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? SB_OK : SB_ERR_LAUNCH + (int)e;
}

// ---------------------------------------------------------------------------------------------
// residency cache of the persistent launchers (declared in sb_internal.h)
#include <mutex>

hipError_t sb_resident_workgroups(const void *kernel, int threads, int *resident)
{
    struct Entry { const void *kernel; int dev, threads, value; };
    static Entry table[512];
    static int used = 0;
    static std::mutex lock;
    const int dev = sb_current_device();
    std::lock_guard<std::mutex> hold(lock);
    for (int i = 0; i < used; ++i)
        if (table[i].kernel == kernel && table[i].dev == dev && table[i].threads == threads) { *resident = table[i].value; return hipSuccess; }
    int per_cu = 0, cus = 0;
    hipError_t e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, 0);
    if (e != hipSuccess) return e;
    if (per_cu < 1 || cus < 1) return hipErrorInvalidConfiguration;
    *resident = per_cu * cus;
    if (used < 512) table[used++] = Entry{kernel, dev, threads, *resident};
    return hipSuccess;
}
