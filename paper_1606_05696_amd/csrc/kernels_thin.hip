// Thin StridedBatchedGemm kernels: problems in which m or n is at most 4, the BatchedGemv end of
// the primitive (the GEMV and dot-product rows of Table I and the n = 1 / m = 1 evaluations of
// section IV-B are such calls).  They are level-2 work: every element of the large operand is
// used once per result column, so the roofline is the HBM rate at which that operand streams in,
// and matrix cores have nothing to offer.
//
// Both kernels compute, per batch entry,
//     y(r, v) = alpha * sum_l M(r, l) * X(l, v) + beta * y(r, v),   r < R, v < nv <= 4, l < K,
// where M is the large operand (op(A) when n is the thin extent, op(B) transposed when m is) and
// X holds the few vectors.  All operands are addressed by (row stride, column stride), so N, T and
// the extended operations of section III-E are all accepted.
//
//   rows kernel : lanes run along r (M's rows are the fast direction).  A workgroup owns 64*VEC
//                 rows, VEC neighbouring ones per lane; its 4 or 16 waves split l and their
//                 partial sums meet in LDS.  Eight (16-byte) or sixteen (narrower) loads are in flight per lane.
//   dots kernel : lanes run along l (M's columns are the fast direction).  A group of 64 or 16
//                 lanes owns 4 rows, each lane accumulates its share of the 4 dot products, and
//                 a butterfly over the group finishes them.
// VEC > 1 variants read M (and, in the dots kernel, X) as 16-byte (or, bf16 only, 4-byte) vectors;
// they need the fast stride to be 1 and the extent along the vector to be whole vectors (the
// hardware reads a vector at any element-aligned address, so neither the other strides nor the
// base address matter).  VEC = 1 variants take anything.
#include "sb_device.h"
#include "sb_internal.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
// global loads of 16 (4) bytes at any address that is aligned for the element: the hardware takes them
typedef uint32_t u32x4a4 __attribute__((ext_vector_type(4), aligned(4)));
typedef uint32_t u32x4a8 __attribute__((ext_vector_type(4), aligned(8)));
typedef uint32_t u32x4a2 __attribute__((ext_vector_type(4), aligned(2)));
typedef uint32_t u32a2 __attribute__((aligned(2)));

struct Thin {
    const void *M, *X;
    void *Y;
    int64_t R, K;
    int nv;
    int64_t rsM, csM, sxl, sxv, syr, syv;
    int64_t bsM[2], bsX[2], bsY[2];
    int64_t batch0, batch1;
    int64_t xspan;            // elements from X to one past the last element of X any batch entry reads
    double alpha, beta;
};

// VEC consecutive elements of T, loaded raw and converted to the accumulation type at use, so
// that a batch of loads can be issued before the first conversion waits for one of them.
template <typename T, typename Acc, int VEC> struct Pack;

template <typename T, typename Acc> struct Pack<T, Acc, 1> {
    typedef T Raw;
    static __device__ __forceinline__ Raw load(const T *p) { return *p; }
    static __device__ __forceinline__ void unpack(const Raw &r, Acc (&v)[1]) { v[0] = sb_load<T, Acc>(&r); }
};
template <> struct Pack<float, float, 4> {
    typedef u32x4 Raw;
    static __device__ __forceinline__ Raw load(const float *p) { return *(const u32x4a4 *)p; }
    static __device__ __forceinline__ void unpack(const Raw &r, float (&v)[4])
    {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = __uint_as_float(r[e]);
    }
};
template <> struct Pack<double, double, 2> {
    typedef u32x4 Raw;
    static __device__ __forceinline__ Raw load(const double *p) { return *(const u32x4a8 *)p; }
    static __device__ __forceinline__ void unpack(const Raw &r, double (&v)[2])
    {
        v[0] = __hiloint2double((int)r[1], (int)r[0]);
        v[1] = __hiloint2double((int)r[3], (int)r[2]);
    }
};
template <> struct Pack<sb_bf16, float, 8> {
    typedef u32x4 Raw;
    static __device__ __forceinline__ Raw load(const sb_bf16 *p) { return *(const u32x4a2 *)p; }
    static __device__ __forceinline__ void unpack(const Raw &r, float (&v)[8])
    {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[2 * e] = __uint_as_float(r[e] << 16);
            v[2 * e + 1] = __uint_as_float(r[e] & 0xffff0000u);
        }
    }
};

template <> struct Pack<sb_bf16, float, 2> {
    typedef uint32_t Raw;
    static __device__ __forceinline__ Raw load(const sb_bf16 *p) { return *(const u32a2 *)p; }
    static __device__ __forceinline__ void unpack(const Raw &r, float (&v)[2])
    {
        v[0] = __uint_as_float(r << 16);
        v[1] = __uint_as_float(r & 0xffff0000u);
    }
};

template <typename T> struct VecOf;
template <> struct VecOf<float> { static constexpr int value = 4, dword = 1; };      // elements per 16 / 4 bytes
template <> struct VecOf<double> { static constexpr int value = 2, dword = 1; };
template <> struct VecOf<sb_bf16> { static constexpr int value = 8, dword = 2; };

constexpr int THIN_THREADS = 256, THIN_WAVES = 4;        // the dots kernel's workgroup

// Workgroup -> (batch entry, row tile); false when the workgroup lies beyond the problem.
__device__ __forceinline__ bool thin_locate(const Thin &g, int64_t tiles_r, int64_t &b0, int64_t &b1, int64_t &tile)
{
    const int64_t bid = (int64_t)blockIdx.x + (int64_t)gridDim.x * blockIdx.y;
    if (bid >= tiles_r * g.batch0 * g.batch1) return false;
    const int64_t b = bid / tiles_r;
    tile = bid - b * tiles_r;
    b1 = b / g.batch0;
    b0 = b - b1 * g.batch0;
    return true;
}

// An element at an address that is the same in every lane, read through the scalar unit.  The
// scalar unit reads whole dwords, so a bf16 element comes out of the aligned dword around it --
// unless that dword sticks out of the caller's X ([lo, hi): its first or last element on an odd
// boundary), in which case the element alone is read with a 2-byte load.
template <typename T, typename Acc> __device__ __forceinline__ Acc uniform_load(const T *p, const T *, const T *) { return sb_load<T, Acc>(p); }
template <> __device__ __forceinline__ float uniform_load<sb_bf16, float>(const sb_bf16 *p, const sb_bf16 *lo, const sb_bf16 *hi)
{
    const uint32_t odd = (uint32_t)((uintptr_t)p >> 1) & 1u;      // upper half of its dword?
    const sb_bf16 *q = p - odd;                                   // pointer arithmetic keeps the address space
    if (q < lo || q + 2 > hi) return sb_load<sb_bf16, float>(p);
    const uint32_t w = *(const uint32_t *)q;
    return __uint_as_float(odd ? (w & 0xffff0000u) : (w << 16));
}

template <typename T, typename Acc>
__device__ __forceinline__ void thin_store(T *dst, Acc sum, Acc alpha, Acc beta)
{
    Acc v = alpha * sum;
    if (beta != Acc(0)) v += beta * sb_load<T, Acc>(dst);
    sb_store<T, Acc>(dst, v);
}

// ---------------------------------------------------------------------------------------------
// rows kernel: lane <-> VEC neighbouring rows, wave w of WAVES takes l = w, w+WAVES, w+2*WAVES, ...
// WAVES = 16 is for problems with few rows in all: the loads in flight then come from the split
// of l rather than from the number of workgroups.
template <typename T, typename Acc, int NV, int VEC, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void thin_rows_kernel(Thin g, int64_t tiles_r)
{
    // loads in flight per lane: 8 of 16 bytes, 16 of the narrow ones
    constexpr int TR = 64 * VEC, U = VEC * sizeof(T) >= 16 ? 8 : 16, THREADS = 64 * WAVES;
    typedef Pack<T, Acc, VEC> P;
    __shared__ Acc red[NV][TR];

    int64_t b0, b1, tile;
    if (!thin_locate(g, tiles_r, b0, b1, tile)) return;      // whole workgroup leaves together
    const T *M = (const T *)g.M + b0 * g.bsM[0] + b1 * g.bsM[1];
    const T *X = (const T *)g.X + b0 * g.bsX[0] + b1 * g.bsX[1];
    T *Y = (T *)g.Y + b0 * g.bsY[0] + b1 * g.bsY[1];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t r0 = tile * TR + (int64_t)lane * VEC;
    // rows beyond R read row 0 instead (always there) and are dropped at the end
    const T *mp = M + (r0 < g.R ? r0 : 0) * g.rsM;
    int xoff[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) xoff[v] = v < g.nv ? v : g.nv - 1;

    Acc acc[NV][VEC];
#pragma unroll
    for (int v = 0; v < NV; ++v)
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[v][e] = Acc(0);

    auto fma_column = [&](const typename P::Raw &raw, int64_t l) {
        Acc mv[VEC];
        P::unpack(raw, mv);
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const Acc xv = uniform_load<T, Acc>(X + l * g.sxl + xoff[v] * g.sxv, (const T *)g.X, (const T *)g.X + g.xspan);
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[v][e] += mv[e] * xv;
        }
    };

    int64_t l = wave;
    for (; l + (U - 1) * WAVES < g.K; l += U * WAVES) {
        typename P::Raw raw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) raw[u] = P::load(mp + (l + u * WAVES) * g.csM);
#pragma unroll
        for (int u = 0; u < U; ++u) fma_column(raw[u], l + u * WAVES);
    }
    for (; l < g.K; l += WAVES) fma_column(P::load(mp + l * g.csM), l);

    // the waves add their partial sums into LDS one after the other: a fixed order of additions
    for (int w = 0; w < WAVES; ++w) {
        if (wave == w) {
#pragma unroll
            for (int v = 0; v < NV; ++v)
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    Acc &slot = red[v][lane * VEC + e];
                    slot = w == 0 ? acc[v][e] : slot + acc[v][e];
                }
        }
        __syncthreads();
    }

    const Acc alpha = (Acc)g.alpha, beta = (Acc)g.beta;
    for (int idx = threadIdx.x; idx < NV * TR; idx += THREADS) {
        const int v = idx / TR, rr = idx - v * TR;
        const int64_t r = tile * TR + rr;
        if (r >= g.R || v >= g.nv) continue;
        thin_store<T, Acc>(Y + r * g.syr + v * g.syv, red[v][rr], alpha, beta);
    }
}

// ---------------------------------------------------------------------------------------------
// dots kernel: a group of LPR lanes <-> 4 rows, lane <-> every LPR-th vector along l.  LPR = 64
// for long rows; LPR = 16 puts four groups (16 rows) in a wave so that short rows still keep every
// lane busy.  Each group starts its walk along l at another vector and wraps around: rows whose
// stride is a large power of two would otherwise all be read at the same offset at the same time,
// and those addresses share memory channels.
template <typename T, typename Acc, int NV, int VEC, int LPR>
__global__ __launch_bounds__(THIN_THREADS) void thin_dots_kernel(Thin g, int64_t tiles_r)
{
    constexpr int RW = 4, GROUPS = 64 / LPR, TR = RW * GROUPS * THIN_WAVES;
    static_assert(RW * NV <= LPR, "one lane of a group stores each result");
    typedef Pack<T, Acc, VEC> P;

    int64_t b0, b1, tile;
    if (!thin_locate(g, tiles_r, b0, b1, tile)) return;
    const T *M = (const T *)g.M + b0 * g.bsM[0] + b1 * g.bsM[1];
    const T *X = (const T *)g.X + b0 * g.bsX[0] + b1 * g.bsX[1];
    T *Y = (T *)g.Y + b0 * g.bsY[0] + b1 * g.bsY[1];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int group = lane / LPR, lin = lane % LPR;
    if (tile * TR + wave * (RW * GROUPS) >= g.R) return;      // no barrier below: a wave may leave alone
    const int64_t r_base = tile * TR + (wave * GROUPS + group) * RW;

    const T *mp[RW];
#pragma unroll
    for (int j = 0; j < RW; ++j) {
        const int64_t r = r_base + j < g.R ? r_base + j : g.R - 1;
        mp[j] = M + r * g.rsM;
    }
    const T *xp[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) xp[v] = X + (int64_t)(v < g.nv ? v : g.nv - 1) * g.sxv;

    Acc acc[RW][NV];
#pragma unroll
    for (int j = 0; j < RW; ++j)
#pragma unroll
        for (int v = 0; v < NV; ++v) acc[j][v] = Acc(0);

    // trips of LPR vectors; the extent along a vector is a whole number of vectors, so a vector is
    // inside or outside
    const int64_t trips = (g.K + LPR * VEC - 1) / (LPR * VEC);
    int64_t trip = trips > 0 ? (int64_t)((uint64_t)(r_base / RW) % (uint64_t)trips) : 0;
#pragma unroll 2
    for (int64_t it = 0; it < trips; ++it) {
        const int64_t l = (trip * LPR + lin) * VEC;
        trip = trip + 1 == trips ? 0 : trip + 1;
        if (l < g.K) {
            typename P::Raw rm[RW], rx[NV];
#pragma unroll
            for (int j = 0; j < RW; ++j) rm[j] = P::load(mp[j] + l * g.csM);
#pragma unroll
            for (int v = 0; v < NV; ++v) rx[v] = P::load(xp[v] + l * g.sxl);
            Acc xv[NV][VEC];
#pragma unroll
            for (int v = 0; v < NV; ++v) P::unpack(rx[v], xv[v]);
#pragma unroll
            for (int j = 0; j < RW; ++j) {
                Acc mv[VEC];
                P::unpack(rm[j], mv);
#pragma unroll
                for (int v = 0; v < NV; ++v)
#pragma unroll
                    for (int e = 0; e < VEC; ++e) acc[j][v] += mv[e] * xv[v][e];
            }
        }
    }

    // butterfly inside the group: afterwards each of its lanes holds every complete sum; lane
    // j*NV+v of the group stores y(r_base+j, v)
    Acc mine = Acc(0);
#pragma unroll
    for (int j = 0; j < RW; ++j)
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            Acc s = acc[j][v];
#pragma unroll
            for (int off = LPR / 2; off >= 1; off >>= 1) s += __shfl_xor(s, off);
            if (lin == j * NV + v) mine = s;
        }
    if (lin < RW * NV) {
        const int j = lin / NV, v = lin - j * NV;
        const int64_t r = r_base + j;
        if (r < g.R && v < g.nv)
            thin_store<T, Acc>(Y + r * g.syr + v * g.syv, mine, (Acc)g.alpha, (Acc)g.beta);
    }
}

// ---------------------------------------------------------------------------------------------
bool whole_vectors(int64_t x, int vec) { return x % vec == 0; }

Thin thin_view(const SbArgs &a)
{
    Thin t;
    if (a.n <= a.m) {             // the vectors are the columns of op(B)
        t.M = a.A; t.X = a.B;
        t.R = a.m; t.nv = (int)a.n;
        t.rsM = a.rsA; t.csM = a.csA;
        t.sxl = a.rsB; t.sxv = a.csB;
        t.syr = 1; t.syv = a.ldc;
        for (int i = 0; i < 2; ++i) { t.bsM[i] = a.bsA[i]; t.bsX[i] = a.bsB[i]; }
    } else {                      // C^T = op(B)^T op(A)^T: the vectors are the rows of op(A)
        t.M = a.B; t.X = a.A;
        t.R = a.n; t.nv = (int)a.m;
        t.rsM = a.csB; t.csM = a.rsB;
        t.sxl = a.csA; t.sxv = a.rsA;
        t.syr = a.ldc; t.syv = 1;
        for (int i = 0; i < 2; ++i) { t.bsM[i] = a.bsB[i]; t.bsX[i] = a.bsA[i]; }
    }
    t.Y = a.C;
    t.K = a.k;
    for (int i = 0; i < 2; ++i) t.bsY[i] = a.bsC[i];
    t.batch0 = a.batch0; t.batch1 = a.batch1;
    t.alpha = a.alpha; t.beta = a.beta;
    // strides along extents of 1 are never applied: zero them so that they cannot veto vector loads
    if (t.nv == 1) t.sxv = 0;
    if (t.batch0 == 1) t.bsM[0] = t.bsX[0] = t.bsY[0] = 0;
    if (t.batch1 == 1) t.bsM[1] = t.bsX[1] = t.bsY[1] = 0;
    t.xspan = t.K < 1 ? 0 : 1 + (t.K - 1) * t.sxl + (t.nv - 1) * t.sxv + (t.batch0 - 1) * t.bsX[0] + (t.batch1 - 1) * t.bsX[1];
    return t;
}

template <typename Kernel>
hipError_t launch_grid(Kernel kernel, const Thin &t, int64_t tiles_r, int threads, hipStream_t stream)
{
    const int64_t total = tiles_r * t.batch0 * t.batch1;
    if (total <= 0) return hipSuccess;
    const int64_t maxx = sb_max_grid_x(threads);
    const int64_t gx = total < maxx ? total : maxx;
    const int64_t gy = (total + gx - 1) / gx;
    if (gy > 65535) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(kernel, dim3((unsigned)gx, (unsigned)gy), dim3(threads), 0, stream, t, tiles_r);
    return hipGetLastError();
}

template <typename T, typename Acc, int NV, int VEC>
hipError_t launch_rows(const Thin &t, bool many_waves, hipStream_t stream)
{
    const int64_t tiles = (t.R + 64 * VEC - 1) / (64 * VEC);
    if (many_waves) return launch_grid(thin_rows_kernel<T, Acc, NV, VEC, 16>, t, tiles, 64 * 16, stream);
    return launch_grid(thin_rows_kernel<T, Acc, NV, VEC, 4>, t, tiles, 64 * 4, stream);
}

template <typename T, typename Acc, int NV>
hipError_t launch_nv(const Thin &t, hipStream_t stream)
{
    constexpr int VEC = VecOf<T>::value, MID = VecOf<T>::dword;
    const int64_t batch = t.batch0 * t.batch1;
    // lanes along the rows of M unless its columns are the contiguous direction
    const bool rows = t.K <= 1 || (t.R > 1 && t.rsM <= t.csM);
    if (rows) {
        // The widest loads that still leave a workgroup for every compute unit; when the loads
        // in flight are few even so, sixteen waves each split l instead of four.
        auto usable = [&](int vec) {
            return vec == 1 || (t.rsM == 1 && whole_vectors(t.R, vec));
        };
        auto groups = [&](int vec) { return (t.R + 64 * vec - 1) / (64 * vec) * batch; };
        const int vec = usable(VEC) && groups(VEC) >= 256 ? VEC : (usable(MID) && groups(MID) >= 256 ? MID : 1);
        // bytes in flight per compute unit with four waves to a workgroup (256 units, 8 or 16
        // loads per lane): below 64 KiB the chip's memory pipeline is not kept full
        const int64_t load_bytes = 64 * vec * (int64_t)sizeof(T);
        const int64_t in_flight = groups(vec) * 4 * (load_bytes >= 1024 ? 8 : 16) * load_bytes / 256;
        const bool many_waves = in_flight < 64 * 1024 && t.K >= 128;
        if (vec == VEC) return launch_rows<T, Acc, NV, VEC>(t, many_waves, stream);
        if (vec == MID) return launch_rows<T, Acc, NV, MID>(t, many_waves, stream);
        return launch_rows<T, Acc, NV, 1>(t, many_waves, stream);
    }
    const bool vec = t.csM == 1 && t.sxl == 1 && whole_vectors(t.K, VEC);
    // rows of at most 32 loads per lane group go four groups to a wave
    const bool short_rows = t.K <= 32 * (vec ? VEC : 1);
    const int64_t tile_rows = short_rows ? 64 : 16;
    const int64_t tiles = (t.R + tile_rows - 1) / tile_rows;
    if (vec) {
        if (short_rows) return launch_grid(thin_dots_kernel<T, Acc, NV, VEC, 16>, t, tiles, THIN_THREADS, stream);
        return launch_grid(thin_dots_kernel<T, Acc, NV, VEC, 64>, t, tiles, THIN_THREADS, stream);
    }
    if (short_rows) return launch_grid(thin_dots_kernel<T, Acc, NV, 1, 16>, t, tiles, THIN_THREADS, stream);
    return launch_grid(thin_dots_kernel<T, Acc, NV, 1, 64>, t, tiles, THIN_THREADS, stream);
}

template <typename T, typename Acc>
hipError_t launch(const SbArgs &a, hipStream_t stream)
{
    const Thin t = thin_view(a);
    switch (t.nv) {
    case 1: return launch_nv<T, Acc, 1>(t, stream);
    case 2: return launch_nv<T, Acc, 2>(t, stream);
    default: return launch_nv<T, Acc, 4>(t, stream);          // nv = 3 runs with one idle column
    }
}

}  // namespace

bool sb_thin_supports(sb_dtype, const SbArgs &a)
{
    if (a.nx > 0) return false;             // two batch levels here; deeper nests run on the tiled kernels
    const int64_t lo = a.m < a.n ? a.m : a.n;
    return lo >= 1 && lo <= 4;
}

bool sb_thin_preferred(sb_dtype dt, const SbArgs &a)
{
    // Every thin problem, except those the small-matrix kernels are built for: both extents at
    // most 32 and a short k (a long k with few rows is a set of dot products and stays here, and
    // so do rows that are contiguous along k).
    if (!sb_tiny_supports(dt, a) || a.k >= 1024) return true;
    const Thin t = thin_view(a);
    return t.csM == 1 && t.R > 1 && a.k >= 128;       // rows of M contiguous and long enough for a lane group each
}

hipError_t sb_launch_thin(sb_dtype dt, const SbArgs &a, hipStream_t stream)
{
    switch (dt) {
    case SB_F64:  return launch<double, double>(a, stream);
    case SB_F32:  return launch<float, float>(a, stream);
    case SB_BF16: return launch<sb_bf16, float>(a, stream);
    }
    return hipErrorInvalidValue;
}
