// Tiny-matrix StridedBatchedGemm: the batch-dominated, bandwidth-bound regime (m, n <= 32).
//
// Here a single GEMM is far too small to fill a workgroup, and the whole problem moves only a
// few bytes per flop, so the kernel is organised around memory traffic, not around tiles
// (section III-C: many small GEMMs; section IV-B: on a GPU such shapes are governed by the
// number of global memory transactions).  One WAVEFRONT owns one C_p at a time and walks over
// the batch with a grid-wide stride; nothing is staged through LDS and there is no barrier.
//   - Every operand element is fetched from global memory exactly once, by the lane that feeds
//     it to the matrix core: for a k-contiguous operand a lane reads 4 consecutive k of its
//     row/column as one 16- or 32-byte vector, so the 64 lanes of a load instruction together
//     cover one contiguous block of the matrix.
//   - The product uses the 16x16x4 MFMA (4 lane groups x 4 steps = 16 k per round).  Even here
//     the matrix core pays: it needs no cross-lane traffic to form the 16x16 outer products and
//     runs at a fraction of its rate while memory is the limit.
//   - fp32 results are stored as one 16-byte vector per lane (a lane holds 4 consecutive rows of
//     one column); fp64 results are produced transposed so that 16 lanes write 128 contiguous bytes.
//   - Several batches per wave are in flight at once (UNROLL) to cover memory latency.
//   - An operand shared by all batches (batch strides 0, as A is in every order-2 x order-3
//     contraction) is read once per wave and kept in registers when k <= 16.
#include "sb_device.h"
#include "sb_internal.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef double f64x4 __attribute__((ext_vector_type(4)));
// global accesses: the hardware reads and writes these at any element-aligned address
typedef float f32x4u __attribute__((ext_vector_type(4), aligned(4)));
typedef double f64x4u __attribute__((ext_vector_type(4), aligned(8)));

template <typename T> struct TinyMfma;

// v_mfma_f32_16x16x4_f32: operand lane l holds X[l%16][k = l/16]; result slot r is D[4*(l/16) + r][l%16].
template <> struct TinyMfma<float> {
    typedef f32x4 Acc;
    typedef f32x4 Vec4;
    typedef f32x4u Vec4U;
    static constexpr bool SWAP = false;     // lane = column of C, slots = 4 consecutive rows
    static __device__ __forceinline__ void mma(Acc &c, float first, float second)
    {
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(first, second, c, 0, 0, 0);
    }
};

// v_mfma_f64_16x16x4_f64: same operand layout; result slot r is D[l/16 + 4*r][l%16].
template <> struct TinyMfma<double> {
    typedef f64x4 Acc;
    typedef f64x4 Vec4;
    typedef f64x4u Vec4U;
    static constexpr bool SWAP = true;      // computes C^T: lane = row of C, slots = columns h, h+4, ..
    static __device__ __forceinline__ void mma(Acc &c, double first, double second)
    {
        c = __builtin_amdgcn_mfma_f64_16x16x4f64(first, second, c, 0, 0, 0);
    }
};

constexpr int TINY_THREADS = 256;
constexpr int WAVES = TINY_THREADS / 64;

// 4 consecutive-k elements of row/column `rc` of an operand, starting at k0.
// KC: k is contiguous in memory (stride 1) and rows/columns stride by ld; else the reverse.
template <typename T, bool KC>
__device__ __forceinline__ void load_frag(T (&f)[4], const T *p, int64_t ld, int rc, int rc_count, int64_t k0, int64_t kcount, bool vec_ok)
{
    typedef typename TinyMfma<T>::Vec4 Vec4;
    if (KC) {
        const T *src = p + (int64_t)rc * ld + k0;
        if (vec_ok && rc < rc_count && k0 + 4 <= kcount) {
            Vec4 v = *(const typename TinyMfma<T>::Vec4U *)src;
#pragma unroll
            for (int e = 0; e < 4; ++e) f[e] = v[e];
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) f[e] = (rc < rc_count && k0 + e < kcount) ? src[e] : T(0);
        }
    } else {
        const T *src = p + rc + k0 * ld;
#pragma unroll
        for (int e = 0; e < 4; ++e) f[e] = (rc < rc_count && k0 + e < kcount) ? src[e * ld] : T(0);
    }
}

// TM x TN MFMA blocks of 16 x 16 per C_p; U batches in flight per wave.
// PIPE (k > 16): the operands of the next 16 k are requested before the current ones are multiplied,
// two steps in flight instead of one; without it a wavefront's time is one memory latency per step.
template <typename T, int TM, int TN, bool A_KC, bool B_KC, bool HOIST_A, int U, bool PIPE>
__global__ __launch_bounds__(TINY_THREADS) void sbgemm_tiny_kernel(SbArgs g, int vec_a, int vec_b, int vec_c)
{
    typedef TinyMfma<T> MF;
    typedef typename MF::Acc Acc;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int h = lane >> 4, c16 = lane & 15;
    const int64_t total = g.batch0 * g.batch1;
    const int64_t nwaves = (int64_t)gridDim.x * WAVES;
    const int64_t wid = (int64_t)blockIdx.x * WAVES + wave;
    const int64_t ldA = A_KC ? g.rsA : g.csA;          // stride between rows (KC) or between k (else)
    const int64_t ldB = B_KC ? g.csB : g.rsB;
    const int m = (int)g.m, n = (int)g.n;
    const T alpha = (T)g.alpha, beta = (T)g.beta;

    T fa_shared[TM][4];
    if (HOIST_A) {
#pragma unroll
        for (int a = 0; a < TM; ++a)
            load_frag<T, A_KC>(fa_shared[a], (const T *)g.A, ldA, a * 16 + c16, m, 4 * h, g.k, vec_a);
    }

    // U consecutive batches per step: a wave's loads for all of them are issued before any is used
    for (int64_t base = wid * U; base < total; base += nwaves * U) {
        Acc acc[U][TM][TN];
        const T *Ap[U], *Bp[U];
        T *Cp[U];
        bool live[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t b = base + u;
            live[u] = b < total;
            const int64_t bb = live[u] ? b : 0;
            const int64_t b1 = bb / g.batch0, b0 = bb - b1 * g.batch0;
            const SbOff3 o1 = sb_level1(g, b1);
            Ap[u] = (const T *)g.A + b0 * g.bsA[0] + o1.a;
            Bp[u] = (const T *)g.B + b0 * g.bsB[0] + o1.b;
            Cp[u] = (T *)g.C + b0 * g.bsC[0] + o1.c;
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int c = 0; c < TN; ++c)
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[u][a][c][r] = T(0);
        }
        if constexpr (PIPE) {
            T fa[2][U][TM][4], fb[2][U][TN][4];
            // a step beyond k loads nothing and yields zeros
            auto load_step = [&](int s, int64_t k0) __attribute__((always_inline)) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (!live[u]) continue;                 // wave-uniform
#pragma unroll
                    for (int c = 0; c < TN; ++c)
                        load_frag<T, B_KC>(fb[s][u][c], Bp[u], ldB, c * 16 + c16, n, k0 + 4 * h, g.k, vec_b);
#pragma unroll
                    for (int a = 0; a < TM; ++a)
                        load_frag<T, A_KC>(fa[s][u][a], Ap[u], ldA, a * 16 + c16, m, k0 + 4 * h, g.k, vec_a);
                }
            };
            auto mma_step = [&](int s) __attribute__((always_inline)) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (!live[u]) continue;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
#pragma unroll
                        for (int a = 0; a < TM; ++a)
#pragma unroll
                            for (int c = 0; c < TN; ++c) {
                                if (MF::SWAP) MF::mma(acc[u][a][c], fb[s][u][c][e], fa[s][u][a][e]);
                                else          MF::mma(acc[u][a][c], fa[s][u][a][e], fb[s][u][c][e]);
                            }
                }
            };
            load_step(0, 0);
            for (int64_t k0 = 0; k0 < g.k; k0 += 32) {
                load_step(1, k0 + 16);
                mma_step(0);
                load_step(0, k0 + 32);
                mma_step(1);
            }
        } else {
            for (int64_t k0 = 0; k0 < g.k; k0 += 16) {
                T fa[U][TM][4], fb[U][TN][4];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (!live[u]) continue;                 // wave-uniform
#pragma unroll
                    for (int c = 0; c < TN; ++c)
                        load_frag<T, B_KC>(fb[u][c], Bp[u], ldB, c * 16 + c16, n, k0 + 4 * h, g.k, vec_b);
                    if (!HOIST_A) {
#pragma unroll
                        for (int a = 0; a < TM; ++a)
                            load_frag<T, A_KC>(fa[u][a], Ap[u], ldA, a * 16 + c16, m, k0 + 4 * h, g.k, vec_a);
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (!live[u]) continue;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
#pragma unroll
                        for (int a = 0; a < TM; ++a)
#pragma unroll
                            for (int c = 0; c < TN; ++c) {
                                const T av = HOIST_A ? fa_shared[a][e] : fa[u][a][e];
                                if (MF::SWAP) MF::mma(acc[u][a][c], fb[u][c][e], av);
                                else          MF::mma(acc[u][a][c], av, fb[u][c][e]);
                            }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (!live[u]) continue;
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int c = 0; c < TN; ++c) {
                    if (!MF::SWAP) {
                        // lane: column j, rows i..i+3
                        const int j = c * 16 + c16, i = a * 16 + 4 * h;
                        if (j >= n || i >= m) continue;
                        T *dst = Cp[u] + i + (int64_t)j * g.ldc;
                        if (vec_c && i + 4 <= m) {
                            typename MF::Vec4 v;
#pragma unroll
                            for (int r = 0; r < 4; ++r) v[r] = alpha * acc[u][a][c][r];
                            if (beta != T(0)) {
                                typename MF::Vec4 old = *(const typename MF::Vec4U *)dst;
#pragma unroll
                                for (int r = 0; r < 4; ++r) v[r] += beta * old[r];
                            }
                            *(typename MF::Vec4U *)dst = v;
                        } else {
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                if (i + r >= m) continue;
                                T v = alpha * acc[u][a][c][r];
                                if (beta != T(0)) v += beta * dst[r];
                                dst[r] = v;
                            }
                        }
                    } else {
                        // lane: row i, columns h, h+4, h+8, h+12 of the block
                        const int i = a * 16 + c16;
                        if (i >= m) continue;
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int j = c * 16 + h + 4 * r;
                            if (j >= n) continue;
                            T *dst = Cp[u] + i + (int64_t)j * g.ldc;
                            T v = alpha * acc[u][a][c][r];
                            if (beta != T(0)) v += beta * *dst;
                            *dst = v;
                        }
                    }
                }
        }
    }
}

// ONE: one problem per wave at a time (a short batch split into 16 x 16 blocks: as many waves as possible)
template <typename T, int TM, int TN, bool A_KC, bool B_KC, bool ONE = false>
hipError_t launch3(const SbArgs &a, hipStream_t stream)
{
    const int64_t total = a.batch0 * a.batch1;
    constexpr int U = ONE ? 1 : (TM * TN == 1) ? 4 : (TM * TN == 2 ? 2 : 1);
    const bool hoist = (a.bsA[0] == 0 || a.batch0 == 1) && (a.bsA[1] == 0 || a.batch1 == 1) && a.nx == 0 && a.k <= 16;
    // vector accesses need no alignment beyond the element's (leading dimensions and offsets may be odd)
    const int vec_a = A_KC, vec_b = B_KC, vec_c = 1;
    // enough workgroups to fill the chip several waves deep, no more than the work needs
    int64_t groups = (total + (int64_t)WAVES * U - 1) / ((int64_t)WAVES * U);
    const int64_t cap = 256 * 8;
    if (groups > cap) groups = cap;
    if (groups < 1) return hipSuccess;
    dim3 grid((unsigned)groups), block(TINY_THREADS);
    if (hoist && !ONE) hipLaunchKernelGGL((sbgemm_tiny_kernel<T, TM, TN, A_KC, B_KC, true, U, false>), grid, block, 0, stream, a, vec_a, vec_b, vec_c);
    else if (a.k > 16) hipLaunchKernelGGL((sbgemm_tiny_kernel<T, TM, TN, A_KC, B_KC, false, U, true>), grid, block, 0, stream, a, vec_a, vec_b, vec_c);
    else               hipLaunchKernelGGL((sbgemm_tiny_kernel<T, TM, TN, A_KC, B_KC, false, U, false>), grid, block, 0, stream, a, vec_a, vec_b, vec_c);
    return hipGetLastError();
}

template <typename T, int TM, int TN, bool ONE = false>
hipError_t launch2(const SbArgs &a, hipStream_t stream)
{
    const bool a_kc = (a.csA == 1), b_kc = (a.rsB == 1);
    if (a_kc && b_kc)  return launch3<T, TM, TN, true, true, ONE>(a, stream);
    if (a_kc && !b_kc) return launch3<T, TM, TN, true, false, ONE>(a, stream);
    if (!a_kc && b_kc) return launch3<T, TM, TN, false, true, ONE>(a, stream);
    return launch3<T, TM, TN, false, false, ONE>(a, stream);
}

// A short batch of 32-wide matrices leaves most of the chip idle behind a few long chains (32 waves of 32
// dependent MFMA rounds for 32 problems of 32 x 32 x 32).  The 16 x 16 blocks of C_p are independent products
// of a row block of op(A_p) and a column block of op(B_p), i.e. further batch digits: the row half moves A by
// 16 rows and C by 16 elements, the column half moves B by 16 columns and C by 16 columns.  The same kernel
// then runs four times as many waves, each with a quarter of the chain.  Whole blocks only (m, n multiples
// of 16), while the split batch still fits the chip one wave per SIMD.
bool split_into_blocks(const SbArgs &a, int tm, int tn, SbArgs &s)
{
    if (tm * tn == 1 || (tm == 2 && a.m != 32) || (tn == 2 && a.n != 32)) return false;
    if (a.batch0 * a.batch1 > 1024 / (tm * tn)) return false;
    if (a.nx + (tm == 2) + (tn == 2) > SB_MAX_BATCH_LEVELS - 2) return false;
    s = a;
    if (s.nx == 0) s.cnt1 = s.batch1;
    auto digit = [&](int64_t stepA, int64_t stepB, int64_t stepC) {
        const int x = s.nx++;
        s.xcnt[x] = 2;  s.xsA[x] = stepA;  s.xsB[x] = stepB;  s.xsC[x] = stepC;
        s.batch1 *= 2;
    };
    if (tm == 2) { digit(16 * a.rsA, 0, 16);  s.m = 16; }
    if (tn == 2) { digit(0, 16 * a.csB, 16 * a.ldc);  s.n = 16; }
    return true;
}

template <typename T>
hipError_t launch1(const SbArgs &a, hipStream_t stream)
{
    const int tm = a.m > 16 ? 2 : 1, tn = a.n > 16 ? 2 : 1;
    SbArgs blocks;
    if (split_into_blocks(a, tm, tn, blocks)) {
        sb_note_member(SB_MEMBER_TINY_BLOCKS);
        return launch2<T, 1, 1, true>(blocks, stream);
    }
    sb_note_member(SB_MEMBER_TINY_WHOLE);
    if (tm == 1 && tn == 1) return launch2<T, 1, 1>(a, stream);
    if (tm == 2 && tn == 1) return launch2<T, 2, 1>(a, stream);
    if (tm == 1 && tn == 2) return launch2<T, 1, 2>(a, stream);
    return launch2<T, 2, 2>(a, stream);
}

}  // namespace

bool sb_tiny_supports(sb_dtype dt, const SbArgs &a)
{
    if (dt != SB_F32 && dt != SB_F64) return false;
    if (a.k <= 0 || a.m > 32 || a.n > 32) return false;
    const bool a_ok = (a.csA == 1) || (a.rsA == 1);
    const bool b_ok = (a.rsB == 1) || (a.csB == 1);
    return a_ok && b_ok;
}

// One wavefront walks the whole k of its problem, a chain of memory latencies that grows with k
// (about 0.07 us per k at any batch size, two steps of 16 in flight).  With few problems and a long k
// the tiled kernels, whose prefetch runs further ahead, are faster although they pad the small
// matrices to their tiles.  Measured at m = n = 10, k = 512, fp32: 512 problems 36 us here against
// 28 us tiled, 64 problems 38 against 19 (before the second step in flight); at 4096 problems this
// kernel wins, 40 against 184 us.  At m = n = 32 the two meet near k = 2048.
bool sb_tiny_preferred(sb_dtype dt, const SbArgs &a)
{
    const bool few = a.batch0 * a.batch1 <= 512;
    const int64_t long_k = (a.m <= 16 && a.n <= 16) ? 128 : 1024;
    return !(few && a.k >= long_k && sb_mfma_supports(dt, a));
}

hipError_t sb_launch_tiny(sb_dtype dt, const SbArgs &a, hipStream_t stream)
{
    switch (dt) {
    case SB_F32: return launch1<float>(a, stream);
    case SB_F64: return launch1<double>(a, stream);
    default: break;
    }
    return hipErrorInvalidValue;
}
