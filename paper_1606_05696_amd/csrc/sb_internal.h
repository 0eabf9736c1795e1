// Internal interface between the C-ABI front end and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/sbgemm.h"

// One (two-level) StridedBatchedGemm in stride-normal form.  op(A)(i,l) sits at
// A + i*rsA + l*csA, op(B)(l,j) at B + l*rsB + j*csB, C(i,j) at C + i + j*ldc; batch (p,q) adds
// p*bsX[0] + q*bsX[1] to each pointer.  N, T and the extended operations of section III-E are all
// instances of this form.
struct SbArgs {
    const void *A;
    const void *B;
    void *C;
    int64_t m, n, k;
    int64_t rsA, csA, rsB, csB, ldc;
    int64_t bsA[2], bsB[2], bsC[2];
    int64_t batch0, batch1;
    double alpha, beta;
    // Nests deeper than two levels (section III-F, Listing 2 with more loops): the level-1 index q is a
    // mixed-radix number.  Its lowest digit (extent cnt1) is level 1 proper with strides bsX[1]; the
    // nx further digits (extents xcnt[]) are the outer levels with strides xsX[].  batch1 is the
    // product of all these extents, so every kernel still sees two levels; nx == 0 is the plain case.
    int32_t nx;
    int64_t cnt1;
    int64_t xcnt[SB_MAX_BATCH_LEVELS - 2], xsA[SB_MAX_BATCH_LEVELS - 2], xsB[SB_MAX_BATCH_LEVELS - 2], xsC[SB_MAX_BATCH_LEVELS - 2];
};

// element offsets that level-1 index q adds to the three pointers
struct SbOff3 { int64_t a, b, c; };
__host__ __device__ inline SbOff3 sb_level1(const SbArgs &g, int64_t q)
{
    SbOff3 o;
    if (g.nx == 0) {
        o.a = q * g.bsA[1];  o.b = q * g.bsB[1];  o.c = q * g.bsC[1];
        return o;
    }
    int64_t rest = q / g.cnt1;
    const int64_t d1 = q - rest * g.cnt1;
    o.a = d1 * g.bsA[1];  o.b = d1 * g.bsB[1];  o.c = d1 * g.bsC[1];
    for (int x = 0; x < g.nx; ++x) {
        const int64_t up = rest / g.xcnt[x], d = rest - up * g.xcnt[x];
        o.a += d * g.xsA[x];  o.b += d * g.xsB[x];  o.c += d * g.xsC[x];
        rest = up;
    }
    return o;
}

// Each launcher returns a hipError_t (0 = launched).  The *_supports predicates say whether a
// kernel family can run the problem at all; the selector decides whether it should.
hipError_t sb_launch_generic(sb_dtype dt, const SbArgs &a, hipStream_t stream);

bool sb_tiny_supports(sb_dtype dt, const SbArgs &a);
bool sb_tiny_preferred(sb_dtype dt, const SbArgs &a);
hipError_t sb_launch_tiny(sb_dtype dt, const SbArgs &a, hipStream_t stream);

bool sb_thin_supports(sb_dtype dt, const SbArgs &a);            // m or n at most 4: level-2 kernels
bool sb_thin_preferred(sb_dtype dt, const SbArgs &a);
hipError_t sb_launch_thin(sb_dtype dt, const SbArgs &a, hipStream_t stream);

bool sb_mfma_supports(sb_dtype dt, const SbArgs &a);
bool sb_mfma_preferred(sb_dtype dt, const SbArgs &a);
hipError_t sb_launch_mfma(sb_dtype dt, const SbArgs &a, hipStream_t stream);
hipError_t sb_launch_mfma_bf16(const SbArgs &a, hipStream_t stream);   // bf16 member of the MFMA family
bool sb_panel_bf16_supports(const SbArgs &a);             // bf16, k <= 128: the whole-K panel-grid kernel
bool sb_panel_bf16_preferred(const SbArgs &a);
hipError_t sb_launch_panel_bf16(const SbArgs &a, hipStream_t stream);
bool sb_mfma_exa_supports(sb_dtype dt, const SbArgs &a);       // extended op on the first operand (MFMA family)
hipError_t sb_launch_mfma_exa(sb_dtype dt, const SbArgs &a, hipStream_t stream);

// Diagnostics: a launcher whose family has several members says which one it launched (the numbers are listed
// with sb_last_kernel_member in sbgemm.h); the front end resets the note to 0 before every dispatch.
void sb_note_member(int member);

// out-of-place mode permutation of a packed tensor (benchmark baseline: the conventional evaluation's copy)
hipError_t sb_launch_permute(int esize, int order, const int64_t *dims, const int *perm, const void *src, void *dst, hipStream_t stream);

// Estimated run time of `tiles` equal tiles (area and speed relative to a 128 x 128 tile) on the chip's
// 256 compute units: the launchers use it to choose between tile sizes.
double sb_tile_time(int64_t tiles, double area, double gain);

// Workgroups of `kernel` (launched with `threads` lanes and no dynamic LDS) that the current device holds at
// once: occupancy per compute unit x compute units, asked once per (device, kernel) and cached by the
// kernel's address (many instantiations share one function-pointer type, so a table per C++ type would
// hand one kernel another's answer).
hipError_t sb_resident_workgroups(const void *kernel, int threads, int *resident);

// A launch may not have more than 2^32 - 1 work-items along x: the most workgroups of `threads`
// lanes a one-dimensional grid can hold.  Launchers that take one workgroup per tile either spill
// into y beyond it or leave larger problems to another family.
inline int64_t sb_max_grid_x(int threads) { return (int64_t)0xFFFFFFFFll / threads; }

// Set-up that HIP keeps per device (function attributes, occupancy) is cached per device ordinal in
// std::atomic tables: two host threads that race on a first use both compute the same value.
constexpr int SB_MAX_DEVICES = 64;
inline int sb_current_device()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= SB_MAX_DEVICES) return 0;
    return dev;
}
