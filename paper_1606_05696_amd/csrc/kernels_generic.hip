// General StridedBatchedGemm kernel: any operation (N, T, extended), any strides, any sizes,
// any alpha/beta, fp64 / fp32 / bf16.  It is the path for every shape the specialised kernels
// do not take, and the only one that runs the extended operations of section III-E.
//
// One workgroup of 256 lanes computes a 64 x 64 tile of one C_p (Listing 1, section III-D); the
// batch index is folded into the grid, so the batch loop of the listing costs no host work.
// A 64 x 16 panel of op(A) and a 16 x 64 panel of op(B) are staged through LDS; the global reads
// run along whichever of the two matrix dimensions has the smaller stride so that they coalesce
// for N and for T operands alike.
#include "sb_device.h"
#include "sb_internal.h"

namespace {

constexpr int GM = 64, GN = 64, GK = 16, GPAD = 4;

template <typename T, typename Acc>
__global__ __launch_bounds__(256) void sbgemm_generic_kernel(SbArgs g, int64_t tiles_m, int64_t tiles_n)
{
    __shared__ Acc As[GK][GM + GPAD];
    __shared__ Acc Bs[GK][GN + GPAD];

    const int64_t tiles = tiles_m * tiles_n;
    const int64_t bid = (int64_t)blockIdx.x + (int64_t)gridDim.x * blockIdx.y;
    if (bid >= tiles * g.batch0 * g.batch1) return;          // whole workgroup leaves together
    const int64_t b = bid / tiles, tile = bid - b * tiles;
    const int64_t b1 = b / g.batch0, b0 = b - b1 * g.batch0;
    const SbOff3 o1 = sb_level1(g, b1);
    const int64_t tm = tile % tiles_m, tn = tile / tiles_m;
    const int64_t i0 = tm * GM, j0 = tn * GN;

    const T *A = (const T *)g.A + b0 * g.bsA[0] + o1.a;
    const T *B = (const T *)g.B + b0 * g.bsB[0] + o1.b;
    T *C = (T *)g.C + b0 * g.bsC[0] + o1.c;

    const int t = threadIdx.x;
    const int tx = t & 15, ty = t >> 4;                      // 4 rows x 4 columns per lane
    Acc acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[a][c] = Acc(0);

    // lanes run along rows of op(A) when its row stride is the smaller one, else along k
    const bool a_rows_fast = g.rsA <= g.csA;
    const bool b_cols_fast = g.csB < g.rsB;

    for (int64_t k0 = 0; k0 < g.k; k0 += GK) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            int i, l;
            if (a_rows_fast) { i = t & 63; l = (t >> 6) + 4 * q; }
            else             { l = t & 15; i = (t >> 4) + 16 * q; }
            Acc v = Acc(0);
            if (i0 + i < g.m && k0 + l < g.k) v = sb_load<T, Acc>(A + (i0 + i) * g.rsA + (k0 + l) * g.csA);
            As[l][i] = v;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            int j, l;
            if (b_cols_fast) { j = t & 63; l = (t >> 6) + 4 * q; }
            else             { l = t & 15; j = (t >> 4) + 16 * q; }
            Acc v = Acc(0);
            if (j0 + j < g.n && k0 + l < g.k) v = sb_load<T, Acc>(B + (k0 + l) * g.rsB + (j0 + j) * g.csB);
            Bs[l][j] = v;
        }
        __syncthreads();
#pragma unroll
        for (int l = 0; l < GK; ++l) {
            Acc av[4], bv[4];
#pragma unroll
            for (int a = 0; a < 4; ++a) av[a] = As[l][tx * 4 + a];
#pragma unroll
            for (int c = 0; c < 4; ++c) bv[c] = Bs[l][ty * 4 + c];
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[a][c] += av[a] * bv[c];
        }
        __syncthreads();
    }

    const Acc alpha = (Acc)g.alpha, beta = (Acc)g.beta;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const int64_t j = j0 + ty * 4 + c;
        if (j >= g.n) continue;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const int64_t i = i0 + tx * 4 + a;
            if (i >= g.m) continue;
            T *dst = C + i + j * g.ldc;
            Acc v = alpha * acc[a][c];
            if (beta != Acc(0)) v += beta * sb_load<T, Acc>(dst);
            sb_store<T, Acc>(dst, v);
        }
    }
}

template <typename T, typename Acc>
hipError_t launch(const SbArgs &a, hipStream_t stream)
{
    const int64_t tiles_m = (a.m + GM - 1) / GM, tiles_n = (a.n + GN - 1) / GN;
    const int64_t total = tiles_m * tiles_n * a.batch0 * a.batch1;
    if (total <= 0) return hipSuccess;
    // the x dimension of a grid holds fewer than 2^32 lanes: spill into y
    const int64_t maxx = sb_max_grid_x(256);
    const int64_t gx = total < maxx ? total : maxx;
    const int64_t gy = (total + gx - 1) / gx;
    if (gy > 65535) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((sbgemm_generic_kernel<T, Acc>), dim3((unsigned)gx, (unsigned)gy), dim3(256), 0, stream,
                       a, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace

hipError_t sb_launch_generic(sb_dtype dt, const SbArgs &a, hipStream_t stream)
{
    switch (dt) {
    case SB_F64:  return launch<double, double>(a, stream);
    case SB_F32:  return launch<float, float>(a, stream);
    case SB_BF16: return launch<sb_bf16, float>(a, stream);
    }
    return hipErrorInvalidValue;
}
