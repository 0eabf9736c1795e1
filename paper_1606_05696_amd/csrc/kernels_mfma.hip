// MFMA-tiled StridedBatchedGemm for the large, compute-bound shapes (fp32 and fp64).
//
// One workgroup of four wavefronts computes a 128 x 128 tile of one C_p (Listing 1, section III-D);
// the batch index and the tile index share the grid, so the batch loop costs no host work and
// takes part in the tiling, as the paper argues a strided batch interface allows.  Panels of
// op(A) (128 x BK) and op(B) (BK x 128) are staged through double-buffered LDS with the next
// panel's global loads in flight during the current panel's MFMAs.  Each wave owns a 64 x 64
// sub-tile held in MFMA accumulators.
//
// Column-major C and the MFMA result layout: an MFMA leaves one result COLUMN per lane, so the
// kernel feeds the B fragment as the instruction's first operand and the A fragment as its
// second.  The instruction then produces C^T, whose per-lane column is a run of consecutive
// ROWS of C: a store instruction writes 128 contiguous bytes per half-wave.
//
// Operand layouts in LDS depend on which dimension of the operand is contiguous in memory:
//   k contiguous (A with T, B with N): LDS [row][k]; a lane fetches 16 bytes = several k at once;
//   m/n contiguous (A with N, B with T): LDS [k][row]; a lane fetches one element per k.
// In both cases global loads and LDS stores are 16-byte vectors along the contiguous dimension.
// Within each group of 8 k the lane groups of a wave take interleaved k so that one 16-byte LDS
// read feeds several consecutive MFMAs; the sum over k does not depend on that order.
#include "sb_device.h"
#include "sb_internal.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef double f64x4 __attribute__((ext_vector_type(4)));

template <typename T> struct Mfma;

// v_mfma_f32_32x32x2_f32: operands hold X[l%32][k = l/32]; result slot r of lane l is
// D[8*(r/4) + 4*(l/32) + r%4][l%32].
template <> struct Mfma<float> {
    static constexpr int MI = 32, VEC = 4, NREG = 16;       // 64/MI lane groups x VEC = 8 k per group
    typedef f32x16 Acc;
    typedef float Vec __attribute__((ext_vector_type(4)));
    static __device__ __forceinline__ void mma(Acc &c, float first, float second)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(first, second, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int result_row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }
};

// v_mfma_f64_16x16x4_f64: operands hold X[l%16][k = l/16]; result slot r of lane l is D[l/16 + 4*r][l%16].
template <> struct Mfma<double> {
    static constexpr int MI = 16, VEC = 2, NREG = 4;
    typedef f64x4 Acc;
    typedef double Vec __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ void mma(Acc &c, double first, double second)
    {
        c = __builtin_amdgcn_mfma_f64_16x16x4f64(first, second, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int result_row(int r, int lane) { return (lane >> 4) + 4 * r; }
};

constexpr int NXCD = 8;

// Stage one BK-deep panel (ROWS rows of the operand) from global memory into registers.
// KC: the panel is stored [row][k] with k contiguous in memory (row stride `ld`);
// otherwise rows are contiguous and k strides by `ld`.
template <typename T, bool KC, int ROWS, int BK, int NT>
struct Panel {
    typedef typename Mfma<T>::Vec Vec;
    static constexpr int VEC = Mfma<T>::VEC;
    static constexpr int NVEC = ROWS * BK / VEC / NT;                  // 16-byte vectors per lane
    static constexpr int LDS_LD = (KC ? BK : ROWS) + VEC;              // padded by 16 bytes
    static constexpr int LDS_SIZE = (KC ? ROWS : BK) * LDS_LD;
    static_assert(ROWS * BK % (VEC * NT) == 0, "panel must split evenly over the lanes");

    static __device__ __forceinline__ void coords(int f, int &row, int &k)
    {
        if (KC) { row = f / (BK / VEC); k = (f % (BK / VEC)) * VEC; }
        else    { k = f / (ROWS / VEC); row = (f % (ROWS / VEC)) * VEC; }
    }

    // GUARD = false: the whole panel lies inside the matrix and every vector is 16-byte aligned.
    // GUARD = true: rows_left / k_left say how much of the panel is inside (edge tiles, odd strides).
    template <bool GUARD>
    static __device__ __forceinline__ void load(Vec (&v)[NVEC], const T *p, int64_t ld, int64_t rows_left, int64_t k_left, bool vec_ok)
    {
#pragma unroll
        for (int q = 0; q < NVEC; ++q) {
            int row, k;
            coords((int)threadIdx.x + NT * q, row, k);
            const T *src = KC ? p + (int64_t)row * ld + k : p + (int64_t)k * ld + row;
            if (!GUARD) {
                v[q] = *(const Vec *)src;
                continue;
            }
            const bool inside = KC ? (row < rows_left && k + VEC <= k_left) : (row + VEC <= rows_left && k < k_left);
            if (vec_ok && inside) {
                v[q] = *(const Vec *)src;
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const bool ok = KC ? (row < rows_left && k + e < k_left) : (row + e < rows_left && k < k_left);
                    v[q][e] = ok ? src[e] : T(0);
                }
            }
        }
    }

    static __device__ __forceinline__ void store(T *lds, const Vec (&v)[NVEC])
    {
#pragma unroll
        for (int q = 0; q < NVEC; ++q) {
            int row, k;
            coords((int)threadIdx.x + NT * q, row, k);
            T *dst = KC ? lds + row * LDS_LD + k : lds + k * LDS_LD + row;
            *(Vec *)dst = v[q];
        }
    }

    // Fragment of the MFMA block whose first row is row0, for k-group kg: VEC consecutive MFMA steps.
    static __device__ __forceinline__ void fragment(T (&frag)[VEC], const T *lds, int row0, int kg, int lane)
    {
        constexpr int MI = Mfma<T>::MI;
        const int row = row0 + (lane % MI);
        const int k = kg * 8 + (lane / MI) * VEC;
        if (KC) {
            Vec v = *(const Vec *)(lds + row * LDS_LD + k);
#pragma unroll
            for (int e = 0; e < VEC; ++e) frag[e] = v[e];
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) frag[e] = lds[(k + e) * LDS_LD + row];
        }
    }
};

// Tile configuration: each wave owns WM x WN of C; WAVES_M x WAVES_N waves form the workgroup tile.
template <typename T, bool A_KC, bool B_KC, int BK, int WM, int WN, int WAVES_M, int WAVES_N>
struct Config {
    static constexpr int BM = WM * WAVES_M, BN = WN * WAVES_N;
    static constexpr int NT = 64 * WAVES_M * WAVES_N;
    typedef Mfma<T> MF;
    typedef Panel<T, A_KC, BM, BK, NT> PA;
    typedef Panel<T, B_KC, BN, BK, NT> PB;
    static constexpr int NBM = WM / MF::MI, NBN = WN / MF::MI;         // MFMA blocks per wave tile
};

// The k loop of one tile.  GUARD selects bounds-checked scalar loads (edge tiles, unaligned
// operands) or plain 16-byte vector loads (interior tiles): the latter is branch-free, so the
// compiler can keep the next panel's global loads in flight under the current panel's MFMAs.
template <typename CF, typename T, bool GUARD>
__device__ __forceinline__ void k_loop(typename CF::MF::Acc (&acc)[CF::NBM][CF::NBN], T (*As)[CF::PA::LDS_SIZE], T (*Bs)[CF::PB::LDS_SIZE],
                                        const T *A, const T *B, int64_t ldA, int64_t ldB, int64_t kstepA, int64_t kstepB,
                                        int64_t m_left, int64_t n_left, int64_t K, bool vec_ok, int wm, int wn, int lane, int BKc)
{
    typedef typename CF::MF MF;
    typedef typename CF::PA PA;
    typedef typename CF::PB PB;
    constexpr int MI = MF::MI, VEC = MF::VEC;
    typename PA::Vec ra[PA::NVEC];
    typename PB::Vec rb[PB::NVEC];
    const int64_t nkb = (K + BKc - 1) / BKc;
    PA::template load<GUARD>(ra, A, ldA, m_left, K, vec_ok);
    PB::template load<GUARD>(rb, B, ldB, n_left, K, vec_ok);
    PA::store(As[0], ra);
    PB::store(Bs[0], rb);
    __syncthreads();
    for (int64_t kb = 0; kb < nkb; ++kb) {
        const int cur = (int)(kb & 1);
        const bool more = kb + 1 < nkb;
        if (more) {                                   // next panel's global loads fly during the MFMAs
            const int64_t k0 = (kb + 1) * BKc;
            PA::template load<GUARD>(ra, A + k0 * kstepA, ldA, m_left, K - k0, vec_ok);
            PB::template load<GUARD>(rb, B + k0 * kstepB, ldB, n_left, K - k0, vec_ok);
        }
#pragma unroll
        for (int kg = 0; kg < BKc / 8; ++kg) {
            T fa[CF::NBM][VEC], fb[CF::NBN][VEC];
#pragma unroll
            for (int a = 0; a < CF::NBM; ++a) PA::fragment(fa[a], As[cur], wm + a * MI, kg, lane);
#pragma unroll
            for (int c = 0; c < CF::NBN; ++c) PB::fragment(fb[c], Bs[cur], wn + c * MI, kg, lane);
#pragma unroll
            for (int e = 0; e < VEC; ++e)
#pragma unroll
                for (int a = 0; a < CF::NBM; ++a)
#pragma unroll
                    for (int c = 0; c < CF::NBN; ++c) MF::mma(acc[a][c], fb[c][e], fa[a][e]);   // C^T = B^T A^T
        }
        if (more) {
            PA::store(As[cur ^ 1], ra);
            PB::store(Bs[cur ^ 1], rb);
        }
        __syncthreads();
    }
}

template <typename T, bool A_KC, bool B_KC, int BK, int WM, int WN, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void sbgemm_mfma_kernel(SbArgs g, int tiles_m, int tiles_n, int vec_ok)
{
    typedef Config<T, A_KC, B_KC, BK, WM, WN, WAVES_M, WAVES_N> CF;
    typedef typename CF::MF MF;
    constexpr int MI = MF::MI, BM = CF::BM, BN = CF::BN;
    __shared__ __attribute__((aligned(16))) T As[2][CF::PA::LDS_SIZE];
    __shared__ __attribute__((aligned(16))) T Bs[2][CF::PB::LDS_SIZE];

    // XCD-aware order: hardware hands consecutive workgroup ids to the 8 XCDs in turn; renumber so
    // that each XCD works on a contiguous range of tiles (the tiles of one batch share B_p in its L2)
    const int64_t total = (int64_t)gridDim.x;
    const int64_t bid = blockIdx.x;
    const int64_t q8 = total / NXCD, r8 = total % NXCD;
    const int64_t xcd = bid % NXCD, slot = bid / NXCD;
    const int64_t logical = xcd * q8 + (xcd < r8 ? xcd : r8) + slot;
    const int64_t tiles = (int64_t)tiles_m * tiles_n;
    const int64_t b = logical / tiles;
    const int tile = (int)(logical - b * tiles);
    const int64_t b1 = b / g.batch0, b0 = b - b1 * g.batch0;
    const int tm = tile % tiles_m, tn = tile / tiles_m;
    const int64_t i0 = (int64_t)tm * BM, j0 = (int64_t)tn * BN;

    // op(A)(i,l) = A[i*rsA + l*csA]: with k contiguous the row stride is rsA, else the k stride is csA
    const T *A = (const T *)g.A + b0 * g.bsA[0] + b1 * g.bsA[1] + i0 * g.rsA;
    const T *B = (const T *)g.B + b0 * g.bsB[0] + b1 * g.bsB[1] + j0 * g.csB;
    T *C = (T *)g.C + b0 * g.bsC[0] + b1 * g.bsC[1];
    const int64_t ldA = A_KC ? g.rsA : g.csA;
    const int64_t ldB = B_KC ? g.csB : g.rsB;
    const int64_t kstepA = A_KC ? 1 : g.csA;
    const int64_t kstepB = B_KC ? 1 : g.rsB;
    const int64_t m_left = g.m - i0, n_left = g.n - j0;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave % WAVES_M) * WM, wn = (wave / WAVES_M) * WN;

    typename MF::Acc acc[CF::NBM][CF::NBN];
#pragma unroll
    for (int a = 0; a < CF::NBM; ++a)
#pragma unroll
        for (int c = 0; c < CF::NBN; ++c)
#pragma unroll
            for (int r = 0; r < MF::NREG; ++r) acc[a][c][r] = T(0);

    // workgroup-uniform: interior tile with aligned operands -> branch-free loop
    const bool interior = vec_ok && m_left >= BM && n_left >= BN && (g.k % BK == 0);
    if (interior)
        k_loop<CF, T, false>(acc, As, Bs, A, B, ldA, ldB, kstepA, kstepB, m_left, n_left, g.k, true, wm, wn, lane, BK);
    else
        k_loop<CF, T, true>(acc, As, Bs, A, B, ldA, ldB, kstepA, kstepB, m_left, n_left, g.k, vec_ok, wm, wn, lane, BK);

    // epilogue: lane = row of C within the block, result slot = column
    const T alpha = (T)g.alpha, beta = (T)g.beta;
#pragma unroll
    for (int a = 0; a < CF::NBM; ++a) {
        const int64_t i = i0 + wm + a * MI + (lane % MI);
        if (i >= g.m) continue;
#pragma unroll
        for (int c = 0; c < CF::NBN; ++c) {
#pragma unroll
            for (int r = 0; r < MF::NREG; ++r) {
                const int64_t j = j0 + wn + c * MI + MF::result_row(r, lane);
                if (j >= g.n) continue;
                T *dst = C + i + j * g.ldc;
                T v = alpha * acc[a][c][r];
                if (beta != T(0)) v += beta * *dst;
                *dst = v;
            }
        }
    }
}

template <typename T, int BK, int WM, int WN, int WAVES_M, int WAVES_N>
hipError_t launch(const SbArgs &a, hipStream_t stream)
{
    constexpr int BM = WM * WAVES_M, BN = WN * WAVES_N, NT = 64 * WAVES_M * WAVES_N;
    const int64_t tiles_m = (a.m + BM - 1) / BM, tiles_n = (a.n + BN - 1) / BN;
    const int64_t total = tiles_m * tiles_n * a.batch0 * a.batch1;
    if (total <= 0) return hipSuccess;
    if (total >= (int64_t)1 << 31) return hipErrorInvalidConfiguration;
    constexpr int VEC = Mfma<T>::VEC;
    const bool a_kc = (a.csA == 1), b_kc = (a.rsB == 1);
    auto aligned = [](int64_t v) { return v % VEC == 0; };
    const int vec_ok = ((uintptr_t)a.A % 16 == 0) && ((uintptr_t)a.B % 16 == 0) &&
                       aligned(a_kc ? a.rsA : a.csA) && aligned(b_kc ? a.csB : a.rsB) &&
                       aligned(a.bsA[0]) && aligned(a.bsA[1]) && aligned(a.bsB[0]) && aligned(a.bsB[1]);
    dim3 grid((unsigned)total), block(NT);
    const int tm = (int)tiles_m, tn = (int)tiles_n;
    if (a_kc && b_kc)        hipLaunchKernelGGL((sbgemm_mfma_kernel<T, true, true, BK, WM, WN, WAVES_M, WAVES_N>), grid, block, 0, stream, a, tm, tn, vec_ok);
    else if (a_kc && !b_kc)  hipLaunchKernelGGL((sbgemm_mfma_kernel<T, true, false, BK, WM, WN, WAVES_M, WAVES_N>), grid, block, 0, stream, a, tm, tn, vec_ok);
    else if (!a_kc && b_kc)  hipLaunchKernelGGL((sbgemm_mfma_kernel<T, false, true, BK, WM, WN, WAVES_M, WAVES_N>), grid, block, 0, stream, a, tm, tn, vec_ok);
    else                     hipLaunchKernelGGL((sbgemm_mfma_kernel<T, false, false, BK, WM, WN, WAVES_M, WAVES_N>), grid, block, 0, stream, a, tm, tn, vec_ok);
    return hipGetLastError();
}

}  // namespace

// N and T operands only: one of the two strides of each operand must be 1.
bool sb_mfma_supports(sb_dtype dt, const SbArgs &a)
{
    if (a.k <= 0) return false;
    const bool a_ok = (a.csA == 1) || (a.rsA == 1);
    const bool b_ok = (a.rsB == 1) || (a.csB == 1);
    if (!a_ok || !b_ok) return false;
    // a k-contiguous operand with a single row or a single k is also "row contiguous": either view works
    const int64_t tiles = ((a.m + 63) / 64) * ((a.n + 63) / 64);       // smallest tile used below
    return tiles * a.batch0 * a.batch1 < ((int64_t)1 << 31);
}

bool sb_mfma_preferred(sb_dtype, const SbArgs &a)
{
    return a.m >= 32 && a.n >= 32 && a.k >= 16;
}

hipError_t sb_launch_mfma(sb_dtype dt, const SbArgs &a, hipStream_t stream)
{
    switch (dt) {
    case SB_F32:
        if (a.m <= 64 || a.n <= 64) return launch<float, 16, 32, 32, 2, 2>(a, stream);     // 64 x 64 tiles
        return launch<float, 16, 64, 64, 2, 2>(a, stream);                                  // 128 x 128 tiles
    case SB_F64:
        if (a.m <= 64 || a.n <= 64) return launch<double, 16, 32, 32, 2, 2>(a, stream);
        return launch<double, 16, 64, 32, 2, 4>(a, stream);                                 // 128 x 128 tiles, 8 waves
    case SB_BF16: return sb_launch_mfma_bf16(a, stream);
    default: break;
    }
    return hipErrorInvalidValue;
}
