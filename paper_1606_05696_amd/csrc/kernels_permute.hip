// Out-of-place mode permutation of a packed column-major tensor: the explicit copy step of the
// conventional evaluation of a contraction (section II-D: permute the operands into matricised
// form, one GEMM, permute the result back).  The library's own contraction path never calls it;
// it exists so that benchmarks can price that copy with the same GEMM code on both sides.
//
// dst mode j is src mode perm[j].  Mode 0 of src is contiguous on the way in, mode perm[0] of src
// is contiguous on the way out, so a workgroup moves a 64 x 64 tile over those two modes through
// LDS (both sides coalesced); when perm[0] == 0 it copies runs along mode 0.
#include "sb_internal.h"

namespace {

constexpr int PT = 64;            // tile edge
constexpr int MAXO = SB_MAX_MODES;

struct PermArgs {
    const void *src;
    void *dst;
    int order;
    int b;                        // src mode that becomes dst mode 0 (0: plain copy of runs)
    int64_t dim[MAXO];            // src extents
    int64_t ss[MAXO];             // src stride of src mode i
    int64_t ds[MAXO];             // dst stride of src mode i
    int64_t tiles_a, tiles_b;     // tiles along src mode 0 and src mode b
    int64_t outer;                // product of the other extents
};

template <typename T>
__global__ __launch_bounds__(256) void permute_kernel(PermArgs g)
{
    __shared__ T tile[PT][PT + 1];
    const int64_t bid = (int64_t)blockIdx.x + (int64_t)gridDim.x * blockIdx.y;
    const int64_t per_outer = g.tiles_a * g.tiles_b;
    if (bid >= per_outer * g.outer) return;
    int64_t o = bid / per_outer;
    const int64_t t = bid - o * per_outer;
    const int64_t tb = t / g.tiles_a, ta = t - tb * g.tiles_a;
    // offsets of the other modes
    int64_t so = 0, dof = 0;
    for (int i = 1; i < g.order; ++i) {
        if (i == g.b) continue;
        const int64_t idx = o % g.dim[i];
        o /= g.dim[i];
        so += idx * g.ss[i];
        dof += idx * g.ds[i];
    }
    const T *src = (const T *)g.src + so;
    T *dst = (T *)g.dst + dof;
    const int tx = threadIdx.x % PT, ty = threadIdx.x / PT;      // 64 x 4
    const int64_t a0 = ta * PT, b0 = tb * PT;
    if (g.b == 0) {               // mode 0 stays mode 0: rows of up to 64 x 64 consecutive elements
        for (int r = ty; r < PT; r += 4) {
            const int64_t a = a0 * PT + (int64_t)r * PT + tx;
            if (a < g.dim[0]) dst[a] = src[a];
        }
        return;
    }
    const int64_t da = g.dim[0], db = g.dim[g.b];
    for (int r = ty; r < PT; r += 4) {            // read: lanes along src mode 0
        const int64_t a = a0 + tx, b = b0 + r;
        if (a < da && b < db) tile[r][tx] = src[a + b * g.ss[g.b]];
    }
    __syncthreads();
    for (int r = ty; r < PT; r += 4) {            // write: lanes along src mode b (dst mode 0)
        const int64_t a = a0 + r, b = b0 + tx;
        if (a < da && b < db) dst[b + a * g.ds[0]] = tile[tx][r];
    }
}

}  // namespace

hipError_t sb_launch_permute(int esize, int order, const int64_t *dims, const int *perm, const void *src, void *dst, hipStream_t stream)
{
    PermArgs g;
    g.src = src;  g.dst = dst;  g.order = order;
    int64_t s = 1;
    for (int i = 0; i < order; ++i) { g.dim[i] = dims[i]; g.ss[i] = s; s *= dims[i]; }
    if (s == 0) return hipSuccess;
    int64_t d = 1;
    for (int j = 0; j < order; ++j) { g.ds[perm[j]] = d; d *= dims[perm[j]]; }
    g.b = perm[0];
    g.outer = 1;
    for (int i = 1; i < order; ++i)
        if (i != g.b) g.outer *= dims[i];
    if (g.b == 0) { g.tiles_a = (dims[0] + (int64_t)PT * PT - 1) / ((int64_t)PT * PT); g.tiles_b = 1; }
    else          { g.tiles_a = (dims[0] + PT - 1) / PT; g.tiles_b = (dims[g.b] + PT - 1) / PT; }
    const int64_t total = g.tiles_a * g.tiles_b * g.outer;
    const int64_t maxx = sb_max_grid_x(256);
    const int64_t gx = total < maxx ? total : maxx, gy = (total + gx - 1) / gx;
    if (gy > 65535) return hipErrorInvalidConfiguration;
    const dim3 grid((unsigned)gx, (unsigned)gy), block(256);
    switch (esize) {
    case 8: hipLaunchKernelGGL(permute_kernel<uint64_t>, grid, block, 0, stream, g); break;
    case 4: hipLaunchKernelGGL(permute_kernel<uint32_t>, grid, block, 0, stream, g); break;
    case 2: hipLaunchKernelGGL(permute_kernel<uint16_t>, grid, block, 0, stream, g); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}
