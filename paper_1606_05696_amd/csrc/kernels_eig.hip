// Symmetric eigensolver for the Tucker decomposition (Algorithm 1, section II-C): the "leading left
// singular vectors" of an unfolding are the leading eigenvectors of a Gram matrix, which this
// file diagonalises with two-sided Jacobi rotations in the parallel (round-robin) ordering:
// a step rotates n/2 disjoint index pairs (p,q) at once, A <- J^T A J, V <- V J, and n-1 steps
// (a sweep) visit every pair once.  With all pairs of a step disjoint, the 2 x 2 block of A at
// (pair P, pair Q) depends only on its own four elements and on the rotations of P and Q, so a
// step is a fully parallel element-wise update.
//
// Two drivers share the arithmetic: one workgroup holding A and V in LDS for small matrices (the
// 100 x 100 Gram matrices of the iteration), and one launch per step on ping-pong buffers in
// global memory for larger ones (the initialisation).  Neither synchronises with the host: the
// number of sweeps is fixed by the caller.
#include "sb_internal.h"

#include <atomic>

namespace {

// round-robin tournament on ne (even) players: pair t of round r
__device__ __forceinline__ void pair_of(int t, int round, int ne, int &p, int &q)
{
    const int mod = ne - 1;
    if (t == 0) { p = ne - 1; q = round; }
    else {
        p = round + t; if (p >= mod) p -= mod;
        q = round - t; if (q < 0) q += mod;
    }
}

// Jacobi rotation J = [[c, s], [-s, c]] that annihilates the off-diagonal element of
// [[app, apq], [apq, aqq]] under J^T . J; the smaller root of t^2 + 2 theta t - 1 = 0 keeps the
// rotation angle below 45 degrees.
template <typename T>
__device__ __forceinline__ void rotation(T app, T aqq, T apq, T &c, T &s)
{
    if (apq == T(0)) { c = T(1); s = T(0); return; }
    const T theta = (aqq - app) / (T(2) * apq);
    const T t = (theta >= T(0) ? T(1) : T(-1)) / (fabs(theta) + sqrt(theta * theta + T(1)));
    c = T(1) / sqrt(t * t + T(1));
    s = t * c;
}

// The same rotation from the hardware's reciprocal, square root and reciprocal square root (1 ulp
// each) for the in-LDS solver, where one wave computes a round's rotations while fifteen wait for it:
// an inexact angle leaves a remainder far below the threshold, and c^2 + s^2 = c^2 (1 + t^2) is off
// by 2 ulp at most, the same order as the rounding of the exact formula.
__device__ __forceinline__ void rotation_quick(float app, float aqq, float apq, float &c, float &s)
{
    const float theta = (aqq - app) * __builtin_amdgcn_rcpf(2.0f * apq);
    const float t = copysignf(__builtin_amdgcn_rcpf(fabsf(theta) + __builtin_amdgcn_sqrtf(theta * theta + 1.0f)), theta);
    c = __builtin_amdgcn_rsqf(t * t + 1.0f);
    s = t * c;
}
__device__ __forceinline__ void rotation_quick(double app, double aqq, double apq, double &c, double &s) { rotation(app, aqq, apq, c, s); }

// Global-memory step: Ain/Vin -> Aout/Vout (ping-pong, so every thread sees the matrix as it was
// before the step).  n is the matrix order, ne = n rounded up to even (the phantom index of an
// odd matrix pairs with nothing).  Work items: (ne/2)^2 blocks of A, then n * ne/2 row pairs of V.
template <typename T>
__global__ __launch_bounds__(256) void jacobi_step_kernel(const T *__restrict__ Ain, T *__restrict__ Aout,
                                                          const T *__restrict__ Vin, T *__restrict__ Vout, int n, int ne, int round,
                                                          int64_t stride)
{
    // several problems of the same order at a fixed stride: blockIdx.y picks one
    Ain += blockIdx.y * stride; Aout += blockIdx.y * stride;
    Vin += blockIdx.y * stride; Vout += blockIdx.y * stride;
    const int h = ne / 2;
    const int64_t nA = (int64_t)h * h, total = nA + (int64_t)n * h;
    for (int64_t item = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; item < total; item += (int64_t)gridDim.x * blockDim.x) {
        if (item < nA) {
            const int P = (int)(item % h), Q = (int)(item / h);
            int p1, q1, p2, q2;
            pair_of(P, round, ne, p1, q1);
            pair_of(Q, round, ne, p2, q2);
            T cP = T(1), sP = T(0), cQ = T(1), sQ = T(0);
            const bool vP = p1 < n && q1 < n, vQ = p2 < n && q2 < n;
            if (vP) rotation(Ain[p1 + (int64_t)p1 * n], Ain[q1 + (int64_t)q1 * n], Ain[p1 + (int64_t)q1 * n], cP, sP);
            if (vQ) rotation(Ain[p2 + (int64_t)p2 * n], Ain[q2 + (int64_t)q2 * n], Ain[p2 + (int64_t)q2 * n], cQ, sQ);
            const bool rp = p1 < n, rq = q1 < n, cp = p2 < n, cq = q2 < n;
            const T a = (rp && cp) ? Ain[p1 + (int64_t)p2 * n] : T(0), b = (rp && cq) ? Ain[p1 + (int64_t)q2 * n] : T(0);
            const T c = (rq && cp) ? Ain[q1 + (int64_t)p2 * n] : T(0), d = (rq && cq) ? Ain[q1 + (int64_t)q2 * n] : T(0);
            const T x00 = cP * a - sP * c, x01 = cP * b - sP * d;        // J_P^T M
            const T x10 = sP * a + cP * c, x11 = sP * b + cP * d;
            if (rp && cp) Aout[p1 + (int64_t)p2 * n] = x00 * cQ - x01 * sQ;   // . J_Q
            if (rp && cq) Aout[p1 + (int64_t)q2 * n] = x00 * sQ + x01 * cQ;
            if (rq && cp) Aout[q1 + (int64_t)p2 * n] = x10 * cQ - x11 * sQ;
            if (rq && cq) Aout[q1 + (int64_t)q2 * n] = x10 * sQ + x11 * cQ;
        } else {
            const int64_t it = item - nA;
            const int row = (int)(it % n), Q = (int)(it / n);
            int p2, q2;
            pair_of(Q, round, ne, p2, q2);
            const bool cp = p2 < n, cq = q2 < n;
            T cQ = T(1), sQ = T(0);
            if (cp && cq) rotation(Ain[p2 + (int64_t)p2 * n], Ain[q2 + (int64_t)q2 * n], Ain[p2 + (int64_t)q2 * n], cQ, sQ);
            const T vp = cp ? Vin[row + (int64_t)p2 * n] : T(0), vq = cq ? Vin[row + (int64_t)q2 * n] : T(0);
            if (cp) Vout[row + (int64_t)p2 * n] = vp * cQ - vq * sQ;
            if (cq) Vout[row + (int64_t)q2 * n] = vp * sQ + vq * cQ;
        }
    }
}

// The same step for an even order with the matrix kept in tournament order: the pairs of every
// round are the neighbours (2P, 2P+1) of the stored matrix, and the step writes each row and column
// of A (each column of V) where the next round wants it.  Index 0 stays; the others walk round the
// cycle 1 -> 2 -> 4 -> ... -> n-2 -> n-1 -> n-3 -> ... -> 3 -> 1, so that the neighbours are the
// indices opposite one another on a circle of n-1 places (the circle method: every pair meets once
// in n-1 rounds, after which every index is back where it started, so whole sweeps leave the
// matrix in its original order).  Reads are pairs of neighbours along a column, contiguous across
// the lanes of a wave; the walk moves a row by two places at most, so the writes of a wave still
// fill whole cache lines.  Grid: x covers the row pairs, y = column pair, z = 2 * problem + (0: A, 1: V).
__device__ __forceinline__ int next_place(int e, int n)
{
    if (e == 0) return 0;
    if (e & 1) return e == 1 ? 2 : e - 2;
    return e + 2 <= n - 2 ? e + 2 : n - 1;
}

template <typename T>
__global__ __launch_bounds__(256) void jacobi_step_even_kernel(const T *__restrict__ Ain, T *__restrict__ Aout,
                                                               const T *__restrict__ Vin, T *__restrict__ Vout, int n, int64_t stride)
{
    typedef T T2 __attribute__((ext_vector_type(2), aligned(sizeof(T))));      // any element-aligned address
    const int problem = blockIdx.z >> 1;
    const bool is_v = blockIdx.z & 1;
    Ain += problem * stride;
    const int h = n / 2, Q = blockIdx.y, P = blockIdx.x * blockDim.x + threadIdx.x;
    if (P >= h) return;
    const int64_t col0 = (int64_t)(2 * Q) * n, col1 = col0 + n;
    // the rotation of column pair Q (the same for the whole workgroup)
    T cQ, sQ;
    {
        const T2 d1 = *(const T2 *)(Ain + 2 * Q + col1);                   // (a_pq, a_qq)
        rotation(Ain[2 * Q + col0], d1.y, d1.x, cQ, sQ);
    }
    const int64_t out0 = (int64_t)next_place(2 * Q, n) * n, out1 = (int64_t)next_place(2 * Q + 1, n) * n;
    if (is_v) {
        // rows 2P, 2P+1 of V times J_Q; rows of V stay where they are
        Vin += problem * stride; Vout += problem * stride;
        const T2 vp = *(const T2 *)(Vin + 2 * P + col0), vq = *(const T2 *)(Vin + 2 * P + col1);
        *(T2 *)(Vout + 2 * P + out0) = vp * cQ - vq * sQ;
        *(T2 *)(Vout + 2 * P + out1) = vp * sQ + vq * cQ;
        return;
    }
    Aout += problem * stride;
    T cP, sP;
    {
        const int64_t dcol = (int64_t)(2 * P) * n;
        const T2 d1 = *(const T2 *)(Ain + 2 * P + dcol + n);
        rotation(Ain[2 * P + dcol], d1.y, d1.x, cP, sP);
    }
    const T2 m0 = *(const T2 *)(Ain + 2 * P + col0), m1 = *(const T2 *)(Ain + 2 * P + col1);   // (a, c), (b, d)
    const T x00 = cP * m0.x - sP * m0.y, x01 = cP * m1.x - sP * m1.y;        // J_P^T M
    const T x10 = sP * m0.x + cP * m0.y, x11 = sP * m1.x + cP * m1.y;
    const int r0 = next_place(2 * P, n), r1 = next_place(2 * P + 1, n);
    Aout[r0 + out0] = x00 * cQ - x01 * sQ;                                   // . J_Q
    Aout[r0 + out1] = x00 * sQ + x01 * cQ;
    Aout[r1 + out0] = x10 * cQ - x11 * sQ;
    Aout[r1 + out1] = x10 * sQ + x11 * cQ;
}

template <typename T>
__global__ void identity_kernel(T *V, int n, int64_t stride = 0)
{
    V += blockIdx.y * stride;
    const int64_t total = (int64_t)n * n;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x)
        V[e] = (e % n == e / n) ? T(1) : T(0);
}

// Small matrices: the whole iteration in one workgroup, A and V in LDS, updated in place
// (rotations of a step are computed first, then every 2 x 2 block is rewritten by one thread).
// One compute unit does all the arithmetic, so the step is kept short in instructions: an odd
// matrix is padded with a zero row and column (its phantom index then rotates by the identity
// without any test), the pairs and rotations of a step sit in a small LDS table, and the
// (pair, pair) coordinates of a thread's work items advance by addition.  The iteration ends as
// soon as no off-diagonal element exceeds the threshold, and a round without a rotation costs one
// barrier only.
constexpr int LDS_THREADS = 1024;

// what a step needs to know about one pair: the two indices and the rotation; one LDS read
template <typename T>
struct __attribute__((aligned(16))) PairRec { int p, q; T c, s; };

template <typename T>
size_t jacobi_lds_bytes(int n)
{
    const size_t ne = n + (n & 1);
    return 2 * ne * ne * sizeof(T) + 16 + (ne / 2) * (sizeof(PairRec<T>) + sizeof(int));
}

template <typename T>
__global__ __launch_bounds__(LDS_THREADS) void jacobi_lds_kernel(T *A, T *V, const T *V0, int n, int ne, int sweeps, T rel_tol, int64_t stride)
{
    // several problems of the same order at a fixed stride: one workgroup each
    A += blockIdx.x * stride;
    V += blockIdx.x * stride;
    if (V0) V0 += blockIdx.x * stride;
    extern __shared__ __attribute__((aligned(16))) unsigned char raw[];
    const int h = ne / 2, tid = threadIdx.x;
    T *As = (T *)raw;                    // ne x ne, leading dimension ne
    T *Vs = As + ne * ne;                // ne x ne as well (a zero phantom row keeps row pairs aligned)
    // [h], 16-byte aligned; an offset from the array keeps the pointer in the LDS address space
    // (through an integer it would become a generic pointer, read with the slower flat loads)
    PairRec<T> *rec = (PairRec<T> *)(raw + ((2 * (size_t)ne * ne * sizeof(T) + 15) & ~(size_t)15));
    int *list = (int *)(rec + h);        // [h] the pairs that rotate in this round, in any order
    __shared__ int rotates[3];           // how many pairs of the round rotate?  three counters take turns
    __shared__ T wave_max[LDS_THREADS / 64];
    for (int e = tid; e < ne * ne; e += LDS_THREADS) {
        const int i = e % ne, j = e / ne;
        As[e] = (i < n && j < n) ? A[i + j * n] : T(0);
    }
    // the rotations accumulate onto V0 (the basis the matrix was rotated into beforehand) or onto I
    for (int e = tid; e < ne * ne; e += LDS_THREADS) {
        const int i = e % ne, j = e / ne;
        Vs[e] = (i < n && j < n) ? (V0 ? V0[i + j * n] : (i == j ? T(1) : T(0))) : T(0);
    }
    if (tid < 3) rotates[tid] = 0;
    __syncthreads();
    // off-diagonal elements below rounding level of the largest diagonal element are left alone: they
    // no longer move the eigenvalues, and among (nearly) equal eigenvalues they would rotate noise forever
    __shared__ T tiny_s;
    if (tid == 0) {
        T big = T(0);
        for (int i = 0; i < n; ++i) big = fmax(big, fabs(As[i + i * ne]));
        tiny_s = rel_tol * big;
    }
    __syncthreads();
    const T tiny = tiny_s;
    const int nA = h * h;
    const int P0 = tid % h, Q0 = tid / h, dP = LDS_THREADS % h, dQ = LDS_THREADS / h;
    typedef T T2 __attribute__((ext_vector_type(2)));
    for (int sweep = 0; sweep < sweeps; ++sweep) {
        // Done when no off-diagonal element is above the threshold: one pass over the matrix instead
        // of a sweep that finds nothing to rotate (a warm-started matrix often needs a single sweep).
        T big = T(0);
        for (int e = tid; e < ne * ne; e += LDS_THREADS)
            if (e % ne != e / ne) big = fmax(big, fabs(As[e]));
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) big = fmax(big, __shfl_xor(big, off));
        if ((tid & 63) == 0) wave_max[tid >> 6] = big;
        __syncthreads();
        big = wave_max[0];
#pragma unroll
        for (int w = 1; w < LDS_THREADS / 64; ++w) big = fmax(big, wave_max[w]);
        __syncthreads();                 // wave_max is rewritten by the next sweep's pass
        if (!(big > tiny)) break;        // workgroup-uniform
        for (int round = 0; round < ne - 1; ++round) {
            const int flag = (sweep * (ne - 1) + round) % 3;
            if (tid == 0) rotates[(flag + 1) % 3] = 0;      // the next round's flag; last read two rounds ago
            if (tid < h) {
                int p, q;
                pair_of(tid, round, ne, p, q);
                T c = T(1), s = T(0);
                const T apq = As[p + q * ne];                                       // phantom index: apq = 0 -> identity
                const T app = As[p + p * ne], aqq = As[q + q * ne];                 // read with apq: one LDS latency, not two
                if (fabs(apq) > tiny) {
                    rotation_quick(app, aqq, apq, c, s);
                    if (s != T(0)) list[atomicAdd(&rotates[flag], 1)] = tid;        // on the list <=> s != 0
                    else c = T(1);
                }
                PairRec<T> r;
                r.p = p; r.q = q; r.c = c; r.s = s;
                rec[tid] = r;
            }
            __syncthreads();
            const int k = rotates[flag];
            if (k == 0) continue;                // workgroup-uniform: nothing moves in this round
            // block (P, Q) of A: J_P^T . J_Q
            // (the kernel is bound by vector-instruction issue: 24-bit multiplies run at full rate, 32-bit ones at a quarter)
            auto update_a = [&](const PairRec<T> &rP, const PairRec<T> &rQ) __attribute__((always_inline)) {
                const int p1 = rP.p, q1 = rP.q, p2 = __mul24(rQ.p, ne), q2 = __mul24(rQ.q, ne);
                const T cP = rP.c, sP = rP.s, cQ = rQ.c, sQ = rQ.s;
                const T a = As[p1 + p2], b = As[p1 + q2], c = As[q1 + p2], d = As[q1 + q2];
                const T x00 = cP * a - sP * c, x01 = cP * b - sP * d;
                const T x10 = sP * a + cP * c, x11 = sP * b + cP * d;
                As[p1 + p2] = x00 * cQ - x01 * sQ;
                As[p1 + q2] = x00 * sQ + x01 * cQ;
                As[q1 + p2] = x10 * cQ - x11 * sQ;
                As[q1 + q2] = x10 * sQ + x11 * cQ;
            };
            // rows 2R and 2R+1 of V times J_Q
            auto update_v = [&](int R, const PairRec<T> &rQ) __attribute__((always_inline)) {
                T2 *vp = (T2 *)(Vs + 2 * R + __mul24(rQ.p, ne)), *vq = (T2 *)(Vs + 2 * R + __mul24(rQ.q, ne));
                const T2 up = *vp, uq = *vq;
                *vp = up * rQ.c - uq * rQ.s;
                *vq = up * rQ.s + uq * rQ.c;
            };
            if (8 * k > h) {
                // most blocks change: the whole (P, Q) grid, which serves V as well (row pair P, column pair Q)
                int P = P0, Q = Q0;
                for (int item = tid; item < nA; item += LDS_THREADS) {
                    // every read of the item before its first write: a write might alias any later read
                    // for all the compiler knows, and each read waited for is an LDS latency
                    const PairRec<T> rP = rec[P], rQ = rec[Q];
                    const int p1 = rP.p, q1 = rP.q, p2 = __mul24(rQ.p, ne), q2 = __mul24(rQ.q, ne);
                    const T cP = rP.c, sP = rP.s, cQ = rQ.c, sQ = rQ.s;
                    T2 *vp = (T2 *)(Vs + 2 * P + p2), *vq = (T2 *)(Vs + 2 * P + q2);
                    const T a = As[p1 + p2], b = As[p1 + q2], c = As[q1 + p2], d = As[q1 + q2];
                    const T2 up = *vp, uq = *vq;
                    const T x00 = cP * a - sP * c, x01 = cP * b - sP * d;
                    const T x10 = sP * a + cP * c, x11 = sP * b + cP * d;
                    As[p1 + p2] = x00 * cQ - x01 * sQ;
                    As[p1 + q2] = x00 * sQ + x01 * cQ;
                    As[q1 + p2] = x10 * cQ - x11 * sQ;
                    As[q1 + q2] = x10 * sQ + x11 * cQ;
                    *vp = up * cQ - uq * sQ;
                    *vq = up * sQ + uq * cQ;
                    P += dP; Q += dQ;
                    if (P >= h) { P -= h; ++Q; }
                }
            } else {
                // Few pairs rotate (the later sweeps of a warm start): only the block rows and block
                // columns of A and the column pairs of V that belong to a listed pair change.  Three
                // families of k * h items on a grid of h x 3k: blocks (listed, any), blocks (any that
                // does not rotate, listed) -- a rotating row pair is in the first family already --
                // and V's (row pair, listed).
                int J = P0, I = Q0;
                for (int item = tid; item < 3 * k * h; item += LDS_THREADS) {
                    const int fam = (I >= k) + (I >= 2 * k);
                    const int L = list[I - fam * k];
                    const PairRec<T> rL = rec[L], rJ = rec[J];
                    if (fam == 0) update_a(rL, rJ);
                    else if (fam == 1) { if (rJ.s == T(0)) update_a(rJ, rL); }
                    else update_v(J, rL);
                    J += dP; I += dQ;
                    if (J >= h) { J -= h; ++I; }
                }
            }
            __syncthreads();
        }
    }
    for (int e = tid; e < n * n; e += LDS_THREADS) {
        A[e] = As[e % n + (e / n) * ne];
        V[e] = Vs[e % n + (e / n) * ne];
    }
}

// Order the eigenvalues (the diagonal of the rotated matrix): rank[i] = number of eigenvalues that
// come before lambda_i in descending order (ties by index); lam[rank] = lambda_i, sel[rank] = i.
template <typename T>
__global__ __launch_bounds__(256) void eig_order_kernel(const T *A, int n, T *lam, int *sel, int64_t stride, int64_t stride_sel)
{
    A += blockIdx.y * stride;
    lam += blockIdx.y * stride;
    sel += blockIdx.y * stride_sel;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
        const T li = A[i + (int64_t)i * n];
        int rank = 0;
        for (int j = 0; j < n; ++j) {
            const T lj = A[j + (int64_t)j * n];
            rank += (lj > li) || (lj == li && j < i);
        }
        lam[rank] = li;
        sel[rank] = i;
    }
}

// W[:, c] = V[:, sel[c]] * scale_c for the r leading eigenpairs; scale_c = 1 (scaled == 0) or
// 1/sqrt(lambda_c), the factor that turns an eigenvector of Y^T Y into Y^T u (zero when the
// eigenvalue is not safely positive: a rank-deficient matrix has no such singular vector).
template <typename T>
__global__ __launch_bounds__(256) void eig_gather_kernel(const T *V, int n, const int *sel, const T *lam, int r, T *W, int64_t ldw, int scaled, T floor_rel)
{
    const int64_t total = (int64_t)n * r;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int row = (int)(e % n), c = (int)(e / n);
        T scale = T(1);
        if (scaled) scale = (lam[c] > floor_rel * lam[0] && lam[c] > T(0)) ? T(1) / sqrt(lam[c]) : T(0);
        int col = sel[c];
        if ((unsigned)col >= (unsigned)n) col = 0;         // NaN eigenvalues leave the order undefined; stay in bounds
        W[row + c * ldw] = V[row + (int64_t)col * n] * scale;
    }
}

template <typename T>
hipError_t eig_impl(int n, int count, int64_t stride_bytes, T *A, T *A2, T *V, T *V2, const T *V0, T *lam, int *sel, int sweeps,
                    hipStream_t stream, T **A_final, T **V_final)
{
    const int ne = n + (n & 1);
    const int64_t stride = stride_bytes / (int64_t)sizeof(T), stride_sel = stride_bytes / (int64_t)sizeof(int);
    if (count < 1 || (count > 1 && (V0 || n == 1))) return hipErrorInvalidValue;      // batches start from the identity
    if (n == 1) {
        if (V0) { hipError_t e = hipMemcpyAsync(V, V0, sizeof(T), hipMemcpyDeviceToDevice, stream); if (e != hipSuccess) return e; }
        else identity_kernel<T><<<1, 64, 0, stream>>>(V, 1);
        *A_final = A; *V_final = V;
    } else if (jacobi_lds_bytes<T>(n) <= (size_t)160 * 1024 - 512) {      // 512 bytes stay for the static variables
        const size_t bytes = jacobi_lds_bytes<T>(n);
        static std::atomic<bool> configured[SB_MAX_DEVICES] = {};
        const int dev = sb_current_device();
        if (!configured[dev]) {
            hipError_t e = hipFuncSetAttribute((const void *)jacobi_lds_kernel<T>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 512);
            if (e != hipSuccess) return e;
            configured[dev] = true;
        }
        // 8 units of rounding of the largest diagonal element: rotating smaller elements only stirs rounding
        // noise (each sweep creates as much as it removes), and a warm-started solve would never stop early
        const T rel_tol = sizeof(T) == 8 ? T(1.8e-15) : T(9.6e-7);
        jacobi_lds_kernel<T><<<count, LDS_THREADS, bytes, stream>>>(A, V, V0, n, ne, sweeps, rel_tol, stride);
        *A_final = A; *V_final = V;
    } else {
        const int h = ne / 2;
        const int64_t items = (int64_t)h * h + (int64_t)n * h;
        const unsigned blocks = (unsigned)((items + 255) / 256 < 4096 ? (items + 255) / 256 : 4096);
        if (V0) { hipError_t e = hipMemcpyAsync(V, V0, sizeof(T) * n * n, hipMemcpyDeviceToDevice, stream); if (e != hipSuccess) return e; }
        else identity_kernel<T><<<dim3(256, count), 256, 0, stream>>>(V, n, stride);
        T *ain = A, *aout = A2, *vin = V, *vout = V2;
        // an even order takes the step that keeps the matrix in tournament order (n/2 <= 65535 column pairs:
        // any order that fits an int-indexed matrix)
        const bool even = n == ne && h <= 65535;
        const unsigned even_threads = (unsigned)(h < 256 ? (h + 63) / 64 * 64 : 256);
        const dim3 even_grid((unsigned)((h + even_threads - 1) / even_threads), (unsigned)h, (unsigned)(2 * count));
        for (int sweep = 0; sweep < sweeps; ++sweep)
            for (int round = 0; round < ne - 1; ++round) {
                if (even) jacobi_step_even_kernel<T><<<even_grid, even_threads, 0, stream>>>(ain, aout, vin, vout, n, stride);
                else jacobi_step_kernel<T><<<dim3(blocks, count), 256, 0, stream>>>(ain, aout, vin, vout, n, ne, round, stride);
                T *t = ain; ain = aout; aout = t;
                t = vin; vin = vout; vout = t;
            }
        *A_final = ain; *V_final = vin;
    }
    eig_order_kernel<T><<<dim3((n + 255) / 256, count), 256, 0, stream>>>(*A_final, n, lam, sel, stride, stride_sel);
    return hipGetLastError();
}

// Sign convention for a factor matrix: every column is scaled by +-1 so that its entry of largest
// magnitude (the first one among equals) is positive.  One workgroup per column.
template <typename T>
__global__ __launch_bounds__(256) void column_signs_kernel(T *U, int64_t rows, int64_t ld)
{
    __shared__ T best_v[256];
    __shared__ int64_t best_i[256];
    T *col = U + (int64_t)blockIdx.x * ld;
    T bv = T(-1);
    int64_t bi = 0;
    for (int64_t i = threadIdx.x; i < rows; i += 256) {
        const T a = fabs(col[i]);
        if (a > bv) { bv = a; bi = i; }            // ascending i per thread: the first of equals stays
    }
    best_v[threadIdx.x] = bv;
    best_i[threadIdx.x] = bi;
    __syncthreads();
    for (int half = 128; half >= 1; half >>= 1) {
        if ((int)threadIdx.x < half) {
            const T ov = best_v[threadIdx.x + half];
            const int64_t oi = best_i[threadIdx.x + half];
            if (ov > best_v[threadIdx.x] || (ov == best_v[threadIdx.x] && oi < best_i[threadIdx.x])) {
                best_v[threadIdx.x] = ov;
                best_i[threadIdx.x] = oi;
            }
        }
        __syncthreads();
    }
    const bool flip = best_v[0] > T(0) && col[best_i[0]] < T(0);
    __syncthreads();                               // everyone has read the pivot before anyone flips it
    if (flip)
        for (int64_t i = threadIdx.x; i < rows; i += 256) col[i] = -col[i];
}

}  // namespace

// U (rows x r, leading dimension ld): columns scaled by +-1 to the sign convention above.
hipError_t sb_column_signs(sb_dtype dt, void *U, int64_t rows, int64_t r, int64_t ld, hipStream_t stream)
{
    if (rows <= 0 || r <= 0) return hipSuccess;
    if (dt == SB_F64) column_signs_kernel<double><<<(unsigned)r, 256, 0, stream>>>((double *)U, rows, ld);
    else if (dt == SB_F32) column_signs_kernel<float><<<(unsigned)r, 256, 0, stream>>>((float *)U, rows, ld);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

// S[e] = sum over c < count of P[c * elems + e]: the partial Gram matrices of a sum that was split
// to fill the chip are added up in a fixed order (no atomics, so the result is reproducible).
template <typename T>
__global__ __launch_bounds__(256) void sum_slices_kernel(const T *__restrict__ P, T *__restrict__ S, int64_t elems, int count)
{
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < elems; e += (int64_t)gridDim.x * blockDim.x) {
        T acc = P[e];
        for (int c = 1; c < count; ++c) acc += P[(int64_t)c * elems + e];
        S[e] = acc;
    }
}

hipError_t sb_sum_slices(sb_dtype dt, const void *P, void *S, int64_t elems, int count, hipStream_t stream)
{
    if (elems <= 0 || count < 1) return hipErrorInvalidValue;
    const unsigned blocks = (unsigned)((elems + 255) / 256 < 2048 ? (elems + 255) / 256 : 2048);
    if (dt == SB_F64) sum_slices_kernel<double><<<blocks, 256, 0, stream>>>((const double *)P, (double *)S, elems, count);
    else if (dt == SB_F32) sum_slices_kernel<float><<<blocks, 256, 0, stream>>>((const float *)P, (float *)S, elems, count);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

// Eigen-decomposition of the symmetric n x n matrix in A (column-major, packed; destroyed).
// A2, V, V2: n*n elements each; lam: n; sel: n ints.  On return *V_final (V or V2) holds the
// eigenvectors as columns in rotation order, lam the eigenvalues in descending order and sel the
// column of *V_final that belongs to each.  V0 (may be null; not V or V2): the rotations accumulate
// onto this matrix instead of the identity, so for A = V0^T S V0 the result holds eigenvectors of S.
// count > 1: that many independent problems of the same order, every array of problem q lying
// q * stride_bytes after problem 0's (a multiple of 8); they share each launch, V0 must be null.
hipError_t sb_eig_sym(sb_dtype dt, int n, int count, int64_t stride_bytes, void *A, void *A2, void *V, void *V2, const void *V0,
                      void *lam, int *sel, int sweeps, hipStream_t stream, void **A_final, void **V_final)
{
    if (dt == SB_F64) return eig_impl<double>(n, count, stride_bytes, (double *)A, (double *)A2, (double *)V, (double *)V2, (const double *)V0, (double *)lam, sel, sweeps, stream, (double **)A_final, (double **)V_final);
    if (dt == SB_F32) return eig_impl<float>(n, count, stride_bytes, (float *)A, (float *)A2, (float *)V, (float *)V2, (const float *)V0, (float *)lam, sel, sweeps, stream, (float **)A_final, (float **)V_final);
    return hipErrorInvalidValue;
}

// W (n x r, leading dimension ldw) = the r leading eigenvectors, optionally scaled by lambda^-1/2.
hipError_t sb_eig_gather(sb_dtype dt, int n, const void *V, const int *sel, const void *lam, int r, void *W, int64_t ldw, int scaled, hipStream_t stream)
{
    const int64_t total = (int64_t)n * r;
    const unsigned blocks = (unsigned)((total + 255) / 256 < 1024 ? (total + 255) / 256 : 1024);
    if (total == 0) return hipSuccess;
    if (dt == SB_F64) eig_gather_kernel<double><<<blocks, 256, 0, stream>>>((const double *)V, n, sel, (const double *)lam, r, (double *)W, ldw, scaled, 1e-24);
    else if (dt == SB_F32) eig_gather_kernel<float><<<blocks, 256, 0, stream>>>((const float *)V, n, sel, (const float *)lam, r, (float *)W, ldw, scaled, 1e-10f);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}
