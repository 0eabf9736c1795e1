// MFMA kernel for the extended operation on the first operand (section III-E): the batched mode is
// the FIRST, unit-stride mode of the tensor, so each batch's matrix is strided in rows and columns,
//     op(A_b)(i,l) = A[b + i*rs + l*cs],        C_b(i,j) = C[b*strideC + i + j*ldc].
// This is the kernel section III-E asks for (an extended-transpose implementation has to tile the
// tensor in all three of its modes on its way into cache): reading one batch at a time would use one
// element per cache line, so a workgroup takes a 3-D brick of the tensor instead, PB consecutive batches x
// MB rows x BK columns, which is read along b (contiguous runs of PB elements) and, because the
// brick holds MB consecutive rows of every batch, written along i (contiguous runs of MB
// elements of every C_b).  The brick's PB*MB (batch,row) pairs are simply the rows of one MFMA
// tile: all PB batches share the same B panel, so the PB small products are one tall GEMM.
// The transposition between "b contiguous" and "i contiguous" happens for free in the LDS
// addressing of the MFMA fragments (lanes run along i, the panel is stored with b fastest).
//
// The extended operation on the SECOND operand is the same kernel on the transposed problem,
//     C_b^T = op(B_b)^T op(A)^T,
// whose first operand is the strided one: the launcher swaps the operands and the kernel (CT) writes
// its tile transposed, C_b(i,j) at i + j*ldc with i the tile's COLUMN.  The MFMA operands trade places
// so that lanes still run along the unit-stride direction of C.
#include <type_traits>

#include "sb_device.h"
#include "sb_internal.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef double f64x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int NXCD = 8;
constexpr int ET = 256;                 // lanes per workgroup (4 waves)

// Instruction traits (layouts as measured on gfx950): a fragment (Vec) holds VEC consecutive k of row
// l%MI, lane group l/MI taking the next VEC; it is spent in STEPS instructions (one k per lane group
// each for fp32/fp64, all eight at once for bf16).  Result slot r of lane l is
// D[row_lane(l) + row_reg(r)][l%MI].  S is the type the epilogue computes in.
struct ExF32 {
    typedef float T;
    typedef float S;
    typedef f32x16 Acc;
    typedef float Vec __attribute__((ext_vector_type(4)));
    typedef float VecU __attribute__((ext_vector_type(4), aligned(4)));       // global loads: any element address
    static constexpr int MI = 32, VEC = 4, NREG = 16, STEPS = 4;       // 64/MI lane groups along k, VEC k each: 8 k per fragment
    static __device__ __forceinline__ void mma(Acc &c, const Vec &first, const Vec &second, int e) { c = __builtin_amdgcn_mfma_f32_32x32x2f32(first[e], second[e], c, 0, 0, 0); }
    static __device__ __forceinline__ int row_lane(int lane) { return 4 * (lane >> 5); }
    static constexpr int row_reg(int r) { return 8 * (r >> 2) + (r & 3); }
    static __device__ __forceinline__ S to_s(T v) { return v; }
    static __device__ __forceinline__ T from_s(S v) { return v; }
};
struct ExBf16 {
    typedef uint16_t T;                                      // bf16 bits
    typedef float S;
    typedef f32x16 Acc;
    typedef uint16_t Vec __attribute__((ext_vector_type(8)));
    typedef uint16_t VecU __attribute__((ext_vector_type(8), aligned(2)));
    static constexpr int MI = 32, VEC = 8, NREG = 16, STEPS = 1;       // 16 k per fragment, one instruction
    static __device__ __forceinline__ void mma(Acc &c, const Vec &first, const Vec &second, int)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, first), __builtin_bit_cast(bf16x8, second), c, 0, 0, 0);
    }
    static __device__ __forceinline__ int row_lane(int lane) { return 4 * (lane >> 5); }
    static constexpr int row_reg(int r) { return 8 * (r >> 2) + (r & 3); }
    static __device__ __forceinline__ S to_s(T v) { return sb_bf16_to_f32(v); }
    static __device__ __forceinline__ T from_s(S v) { return sb_f32_to_bf16(v); }      // nearest, ties to even
};
struct ExF64 {
    typedef double T;
    typedef double S;
    typedef f64x4 Acc;
    typedef double Vec __attribute__((ext_vector_type(2)));
    typedef double VecU __attribute__((ext_vector_type(2), aligned(8)));
    static constexpr int MI = 16, VEC = 2, NREG = 4, STEPS = 2;
    static __device__ __forceinline__ void mma(Acc &c, const Vec &first, const Vec &second, int e) { c = __builtin_amdgcn_mfma_f64_16x16x4f64(first[e], second[e], c, 0, 0, 0); }
    static __device__ __forceinline__ int row_lane(int lane) { return lane >> 4; }
    static constexpr int row_reg(int r) { return 4 * r; }
    static __device__ __forceinline__ S to_s(T v) { return v; }
    static __device__ __forceinline__ T from_s(S v) { return v; }
};

// PB batches x MB rows per tile (PB*MB tile rows), BN columns, BK deep panels (one group of MFMA
// fragments per panel, or two, so that a barrier comes only every 32 fp32 MFMAs of a wave).
// The second launch bound (waves per SIMD the register allocation must leave room for) keeps two
// fp64 workgroups on a compute unit; left alone the allocator gives the fp64 variant more than 256
// registers and one workgroup per compute unit (35 instead of 54 TFLOP/s at 512^4).  The fp32 variant
// with 16-deep panels takes 212-232 registers by itself, two workgroups per compute unit, and is
// left alone: bounded to three it spills inside the k loop (0.50 instead of 0.70 of the peak), and
// with 8-deep panels three fit but a barrier every 16 MFMAs costs more (0.67).
template <typename MF, bool B_KC, bool CT, int PB, int MB, int BN, int BK>
__global__ __launch_bounds__(ET, sizeof(typename MF::T) == 8 ? 2 : 1) void sbgemm_mfma_exa_kernel(SbArgs g, int tiles_b, int tiles_i, int tiles_n, int vec_a, int vec_b)
{
    typedef typename MF::T T;
    typedef typename MF::Vec Vec;
    typedef typename MF::VecU VecU;
    typedef typename MF::S S;
    constexpr int MI = MF::MI, VEC = MF::VEC, STEPS = MF::STEPS;
    constexpr int KF = (64 / MI) * VEC;               // k per fragment group: 8 (fp32, fp64) or 16 (bf16)
    constexpr int KG = BK / KF;                       // fragment groups per panel
    static_assert(KG == 1 || KG == 2, "one or two fragment groups per panel");
    constexpr int BM = PB * MB;                       // tile rows = (batch, row) pairs
    constexpr int PBP = PB + 16 / (int)sizeof(T);     // b-run padded by 16 bytes: lanes that differ in i hit different banks
    constexpr int A_K = MB * PBP;                     // elements per k slab of the A panel: [k][i][b]
    constexpr int B_LD = B_KC ? BK + VEC : BN + VEC;  // B panel: [col][k] (k contiguous) or [k][col]
    constexpr int B_SIZE = B_KC ? BN * B_LD : BK * B_LD;
    constexpr int NVA = BM * BK / VEC / ET;           // 16-byte vectors of A per lane and panel
    constexpr int NBM = BM / 4 / MI, NBN = BN / MI;   // MFMA blocks per wave: 4 waves split the tile rows
    static_assert(BM * BK % (VEC * ET) == 0 && BM % (4 * MI) == 0 && BN % MI == 0 && PB % VEC == 0, "tile shape");
    static_assert(BN * BK / VEC <= ET, "one vector of B per lane at most");
    __shared__ __attribute__((aligned(16))) T As[2][BK * A_K];
    __shared__ __attribute__((aligned(16))) T Bs[2][B_SIZE];

    // XCD-aware order: consecutive workgroup ids go to the 8 XCDs in turn; renumber so that an XCD
    // owns a contiguous range of tiles.  Column tiles run fastest: the tiles that read the same
    // brick of A are neighbours and share it in one L2.
    const int64_t total = (int64_t)gridDim.x;
    const int64_t bid = blockIdx.x;
    const int64_t q8 = total / NXCD, r8 = total % NXCD;
    const int64_t xcd = bid % NXCD, slot = bid / NXCD;
    int64_t logical = xcd * q8 + (xcd < r8 ? xcd : r8) + slot;
    const int tn = (int)(logical % tiles_n); logical /= tiles_n;
    const int tb = (int)(logical % tiles_b); logical /= tiles_b;
    const int ti = (int)(logical % tiles_i);
    const int64_t b1 = logical / tiles_i;
    const SbOff3 o1 = sb_level1(g, b1);
    const int64_t bb = (int64_t)tb * PB, i0 = (int64_t)ti * MB, j0 = (int64_t)tn * BN;
    const int64_t b_left = g.batch0 - bb, m_left = g.m - i0, n_left = g.n - j0;

    const T *A = (const T *)g.A + bb + o1.a + i0 * g.rsA;        // batch stride of level 0 is 1
    const T *B = (const T *)g.B + o1.b + j0 * g.csB;             // B ignores level 0 here (checked by the launcher)
    const int64_t ldB = B_KC ? g.csB : g.rsB, kstepB = B_KC ? 1 : g.rsB;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    typename MF::Acc acc[NBM][NBN];
#pragma unroll
    for (int a = 0; a < NBM; ++a)
#pragma unroll
        for (int c = 0; c < NBN; ++c)
#pragma unroll
            for (int r = 0; r < MF::NREG; ++r) acc[a][c][r] = S(0);

    // A panel vector f: k = f / (MB * PB/VEC), i = (f / (PB/VEC)) % MB, b = (f % (PB/VEC)) * VEC.
    // FAST: the whole brick lies inside the tensor and is 16-byte aligned (no tests, plain vector loads).
    auto load_a = [&](auto fast_c, Vec (&v)[NVA], int64_t k0) {
#pragma unroll
        for (int q = 0; q < NVA; ++q) {
            const int f = (int)threadIdx.x + ET * q;
            const int k = f / (MB * (PB / VEC)), i = (f / (PB / VEC)) % MB, b = (f % (PB / VEC)) * VEC;
            const T *src = A + b + (int64_t)i * g.rsA + (k0 + k) * g.csA;
            if (decltype(fast_c)::value) {
                v[q] = *(const VecU *)src;
                continue;
            }
            const bool row_ok = i < m_left && k0 + k < g.k;
            if (vec_a && row_ok && b + VEC <= b_left) {
                v[q] = *(const VecU *)src;
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) v[q][e] = (row_ok && b + e < b_left) ? src[e] : T(0);
            }
        }
    };
    auto store_a = [&](T *lds, const Vec (&v)[NVA]) {
#pragma unroll
        for (int q = 0; q < NVA; ++q) {
            const int f = (int)threadIdx.x + ET * q;
            const int k = f / (MB * (PB / VEC)), i = (f / (PB / VEC)) % MB, b = (f % (PB / VEC)) * VEC;
            *(Vec *)(lds + k * A_K + i * PBP + b) = v[q];
        }
    };
    // B panel: one vector per lane for the first BN*BK/VEC lanes
    auto load_b = [&](auto fast_c, Vec &v, int64_t k0) {
        const int f = threadIdx.x;
        if (f >= BN * BK / VEC) return;
        int col, k;
        if (B_KC) { col = f / (BK / VEC); k = (f % (BK / VEC)) * VEC; }
        else      { k = f / (BN / VEC); col = (f % (BN / VEC)) * VEC; }
        const T *src = B_KC ? B + (int64_t)col * ldB + (k0 + k) : B + (k0 + k) * kstepB + col;
        if (decltype(fast_c)::value) {
            v = *(const VecU *)src;
            return;
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const bool ok = B_KC ? (col < n_left && k0 + k + e < g.k) : (col + e < n_left && k0 + k < g.k);
            v[e] = ok ? src[e] : T(0);
        }
    };
    auto store_b = [&](T *lds, const Vec &v) {
        const int f = threadIdx.x;
        if (f >= BN * BK / VEC) return;
        int col, k;
        if (B_KC) { col = f / (BK / VEC); k = (f % (BK / VEC)) * VEC; }
        else      { k = f / (BN / VEC); col = (f % (BN / VEC)) * VEC; }
        *(Vec *)(B_KC ? lds + col * B_LD + k : lds + k * B_LD + col) = v;
    };

    // tile row rho (0 .. BM-1) = (batch rho / MB, row rho % MB): lanes of an MFMA block run along i
    const int rho0 = wave * (BM / 4);
    const int kl = lane / MI;                          // lane group along k
    const int64_t nkb = (g.k + BK - 1) / BK;

    // MFMA operands of one fragment group of a panel (lane group kl takes k = kl*VEC + e)
    auto read_frags = [&](Vec (&fa)[NBM], Vec (&fb)[NBN], int buf, int kg = 0) {
        const int k = kg * KF + kl * VEC;
#pragma unroll
        for (int a = 0; a < NBM; ++a) {
            const int rho = rho0 + a * MI + (lane % MI);
            const T *p = As[buf] + (rho % MB) * PBP + (rho / MB);
#pragma unroll
            for (int e = 0; e < VEC; ++e) fa[a][e] = p[(k + e) * A_K];
        }
#pragma unroll
        for (int c = 0; c < NBN; ++c) {
            const int col = c * MI + (lane % MI);
            if (B_KC) {
                fb[c] = *(const Vec *)(Bs[buf] + col * B_LD + k);
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) fb[c][e] = Bs[buf][(k + e) * B_LD + col];
            }
        }
    };

    // D = first x second^T has lanes along second's rows: tile rows (first = B fragment) when C_b is stored
    // as computed, tile columns when it is stored transposed
    auto mma = [](typename MF::Acc &c, const Vec &row_frag, const Vec &col_frag, int e) {
        if (CT) MF::mma(c, row_frag, col_frag, e);
        else    MF::mma(c, col_frag, row_frag, e);
    };

    // The k loop, software-pipelined like the plain MFMA kernel: global loads run two panels ahead
    // (two staging register sets), the LDS store of the next panel sits in the middle of the MFMA
    // cluster, and the fragments of the next panel are read right after the barrier, before the
    // second half of the current cluster's successor starts.  CUR = parity of the panel.
    Vec ra[2][NVA], rb[2];
    Vec fa[2][NBM], fb[2][NBN];
    auto k_loop = [&](auto fast_c) {
        auto block = [&](auto cur_c, auto steady_c, int64_t kb) {
            constexpr int CUR = decltype(cur_c)::value;
            constexpr bool STEADY = decltype(steady_c)::value;
            if (STEADY || kb + 2 < nkb) {
                load_a(fast_c, ra[CUR], (kb + 2) * BK);
                load_b(fast_c, rb[CUR], (kb + 2) * BK);
            }
            const bool hand_over = STEADY || kb + 1 < nkb;
            if (KG == 2) {
                // Two fragment groups per panel, fragment sets alternate by group: group 1 is read
                // while group 0 is multiplied (with the LDS store of the next panel in the middle
                // of that cluster); the barrier and the next panel's group 0 come before group 1's
                // MFMAs, which then cover both.
                read_frags(fa[1], fb[1], CUR, 1);
                __builtin_amdgcn_s_setprio(2);
#pragma unroll
                for (int e = 0; e < STEPS; ++e) {
                    if (e == STEPS / 2 && hand_over) {
                        __builtin_amdgcn_sched_barrier(0);
                        store_a(As[CUR ^ 1], ra[CUR ^ 1]);
                        store_b(Bs[CUR ^ 1], rb[CUR ^ 1]);
                        __builtin_amdgcn_sched_barrier(0);
                    }
#pragma unroll
                    for (int a = 0; a < NBM; ++a)
#pragma unroll
                        for (int c = 0; c < NBN; ++c) mma(acc[a][c], fa[0][a], fb[0][c], e);
                }
                __builtin_amdgcn_s_setprio(0);
                if (hand_over) {
                    __syncthreads();
                    read_frags(fa[0], fb[0], CUR ^ 1, 0);
                }
                __builtin_amdgcn_s_setprio(2);
#pragma unroll
                for (int e = 0; e < STEPS; ++e)
#pragma unroll
                    for (int a = 0; a < NBM; ++a)
#pragma unroll
                        for (int c = 0; c < NBN; ++c) mma(acc[a][c], fa[1][a], fb[1][c], e);
                __builtin_amdgcn_s_setprio(0);
                return;
            }
            __builtin_amdgcn_s_setprio(2);
#pragma unroll
            for (int e = 0; e < STEPS; ++e) {
                if (e == STEPS / 2 && hand_over) {
                    __builtin_amdgcn_sched_barrier(0);
                    store_a(As[CUR ^ 1], ra[CUR ^ 1]);
                    store_b(Bs[CUR ^ 1], rb[CUR ^ 1]);
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int a = 0; a < NBM; ++a)
#pragma unroll
                    for (int c = 0; c < NBN; ++c) mma(acc[a][c], fa[CUR][a], fb[CUR][c], e);
            }
            __builtin_amdgcn_s_setprio(0);
            if (hand_over) {
                __syncthreads();
                read_frags(fa[CUR ^ 1], fb[CUR ^ 1], CUR ^ 1);
            }
        };
        typedef std::integral_constant<int, 0> I0;
        typedef std::integral_constant<int, 1> I1;
        load_a(fast_c, ra[0], 0);
        load_b(fast_c, rb[0], 0);
        if (nkb > 1) {
            load_a(fast_c, ra[1], BK);
            load_b(fast_c, rb[1], BK);
        }
        store_a(As[0], ra[0]);
        store_b(Bs[0], rb[0]);
        __syncthreads();
        read_frags(fa[0], fb[0], 0);
        int64_t kb = 0;
        for (; kb + 3 < nkb; kb += 2) {
            block(I0(), std::true_type(), kb);
            block(I1(), std::true_type(), kb + 1);
        }
        for (; kb < nkb; kb += 2) {
            block(I0(), std::false_type(), kb);
            if (kb + 1 < nkb) block(I1(), std::false_type(), kb + 1);
        }
    };
    // workgroup-uniform choice
    const bool fast = vec_a && vec_b && b_left >= PB && m_left >= MB && n_left >= BN && g.k % BK == 0;
    if (fast) k_loop(std::true_type());
    else      k_loop(std::false_type());

    // epilogue: lane = tile row rho = (batch, row); consecutive lanes are consecutive rows of one C_b.
    // The variants (whole brick or not, beta or not) are chosen by workgroup-uniform branches so that
    // the common one is a straight run of stores.
    const S alpha = (S)g.alpha, beta = (S)g.beta;
    auto store_tile = [&](auto guard_c, auto beta_c) {
        constexpr bool GUARD = decltype(guard_c)::value, BETA = decltype(beta_c)::value;
        if (CT) {
            // lane = tile column = row of the stored C_b (unit stride); slots run over (batch, tile row) pairs,
            // the tile row being the stored column
#pragma unroll
            for (int c = 0; c < NBN; ++c) {
                const int col = c * MI + (lane % MI);
                if (GUARD && col >= n_left) continue;
                T *Cc = (T *)g.C + o1.c + (j0 + col);
#pragma unroll
                for (int a = 0; a < NBM; ++a)
#pragma unroll
                    for (int r = 0; r < MF::NREG; ++r) {
                        const int rho = rho0 + a * MI + MF::row_lane(lane) + MF::row_reg(r);
                        const int bl = rho / MB, il = rho % MB;
                        if (GUARD && (bl >= b_left || il >= m_left)) continue;
                        T *dst = Cc + (bb + bl) * g.bsC[0] + (i0 + il) * g.ldc;
                        S v = alpha * acc[a][c][r];
                        if (BETA) v += beta * MF::to_s(*dst);
                        *dst = MF::from_s(v);
                    }
            }
            return;
        }
#pragma unroll
        for (int a = 0; a < NBM; ++a) {
            const int rho = rho0 + a * MI + (lane % MI);
            const int bl = rho / MB, il = rho % MB;
            if (GUARD && (bl >= b_left || il >= m_left)) continue;
            T *Cb = (T *)g.C + (bb + bl) * g.bsC[0] + o1.c + (i0 + il);
#pragma unroll
            for (int c = 0; c < NBN; ++c) {
                const int64_t jl = j0 + c * MI + MF::row_lane(lane);
                T *col = Cb + jl * g.ldc;
#pragma unroll
                for (int r = 0; r < MF::NREG; ++r) {
                    if (GUARD && jl + MF::row_reg(r) >= g.n) continue;
                    T *dst = col + MF::row_reg(r) * g.ldc;
                    S v = alpha * acc[a][c][r];
                    if (BETA) v += beta * MF::to_s(*dst);
                    *dst = MF::from_s(v);
                }
            }
        }
    };
    const bool whole = b_left >= PB && m_left >= MB && n_left >= BN;
    if (whole) {
        if (beta == S(0)) store_tile(std::false_type(), std::false_type());
        else              store_tile(std::false_type(), std::true_type());
    } else {
        if (beta == S(0)) store_tile(std::true_type(), std::false_type());
        else              store_tile(std::true_type(), std::true_type());
    }
}

// Direct-to-LDS member (fp32 and fp64, whole bricks): the same brick and the same MFMA tile, but the panels travel
// from memory straight into two LDS stages (global_load_lds_dwordx4: no staging registers, no LDS store
// instructions), one barrier per panel.  LDS cannot be padded by such loads (lane l lands at base + 16 l), so
// the layouts are unpadded and conflicts are avoided by what each lane fetches into its slot:
//   A brick   [k][i][16 b]: the 16-byte chunks of row i (four of 4 batches in fp32, eight of 2 in fp64) sit at
//             chunk ^ f(i), f(i) = (i / 4) % 4 or (i / 2) % 8: the 16 lanes of a fragment read that differ in i
//             then cover 16 different 16-byte columns of the banks;
//   B panel   k contiguous: [col][64 bytes of k], chunk of column col at chunk ^ (col / 4) % 4; otherwise
//             [k][BN columns] as it lies (lanes along the columns).
// A load instruction of a wave fetches one k of the brick (fp64: half of one), so its base pointer carries k and
// the lane offsets stay small.  fp32: 16-deep panels of two fragment groups (the second group is read while the
// first is multiplied, the barrier sits between them), tiles 64 or 128 columns wide (a wave's 64 rows x 128
// columns reuse each A fragment four times); fp64: 8-deep panels of one group, 64 columns, the next panel's
// fragments read ahead of the current panel's MFMAs.  Per panel and wave: five or six loads requested two panels
// ahead, 32 or 64 MFMAs.
template <typename MF, bool B_KC, bool CT, int BN>
__global__ __launch_bounds__(256, 2) void sbgemm_mfma_exa_dma_kernel(SbArgs g, int tiles_b, int tiles_i, int tiles_n)
{
    typedef typename MF::T T;
    typedef typename MF::Vec Vec;
    typedef typename MF::S S;
    constexpr int PB = 16, MB = 16, MI = MF::MI, VEC = MF::VEC, STEPS = MF::STEPS;
    constexpr int KF = (64 / MI) * VEC;               // k per fragment group: 8
    constexpr int BK = 64 / (int)sizeof(T);           // 64 bytes of k per panel: 16 (fp32) or 8 (fp64)
    constexpr int KG = BK / KF;                       // fragment groups per panel: 2 or 1
    constexpr int CPR = PB / VEC;                     // 16-byte chunks of a (k, i) run of 16 batches
    constexpr int RPI = 64 / CPR, IPK = MB / RPI;     // rows i per load instruction, load instructions per k
    constexpr int ISH = sizeof(T) == 4 ? 2 : 1;       // f(i) = (i >> ISH) % CPR
    constexpr int NLB = BN / 64;                      // loads of B per wave and panel (1 KB each)
    constexpr int BM = PB * MB, NBM = BM / 4 / MI, NBN = BN / MI;
    constexpr int A_SIZE = BK * MB * PB, B_SIZE = BN * BK, STAGE = A_SIZE + B_SIZE;       // elements
    static_assert(BK * IPK == 16 && (KG == 1 || KG == 2) && NLB >= 1, "four loads of A per wave and panel");
    // A column-contiguous fp32 B panel lies [k][col]: one LDS read of NBN consecutive columns at one k feeds all
    // NBN MFMA blocks of the wave if lane j of block c stands for tile column NBN j + c (instead of 32 c + j);
    // the column <-> (block, lane) map is free as long as every k uses it.  (Not with the transposed tile write,
    // whose lanes run along these columns when they store.)
    constexpr bool B_IL = !B_KC && !CT && sizeof(T) == 4 && (NBN == 2 || NBN == 4);
    typedef T ColVec __attribute__((ext_vector_type(NBN > 1 ? NBN : 2)));
    __shared__ __attribute__((aligned(16))) T lds[2 * STAGE];

    const int64_t total = (int64_t)gridDim.x;
    const int64_t bid = blockIdx.x;
    const int64_t q8 = total / NXCD, r8 = total % NXCD;
    const int64_t xcd = bid % NXCD, slot = bid / NXCD;
    int64_t logical = xcd * q8 + (xcd < r8 ? xcd : r8) + slot;
    const int tn = (int)(logical % tiles_n); logical /= tiles_n;
    const int tb = (int)(logical % tiles_b); logical /= tiles_b;
    const int ti = (int)(logical % tiles_i);
    const int64_t b1 = logical / tiles_i;
    const SbOff3 o1 = sb_level1(g, b1);
    const int64_t bb = (int64_t)tb * PB, i0 = (int64_t)ti * MB, j0 = (int64_t)tn * BN;
    const T *A = (const T *)g.A + bb + o1.a + i0 * g.rsA;
    const T *B = (const T *)g.B + o1.b + j0 * g.csB;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t nkb = g.k / BK;

    // what this lane fetches (byte offsets from the load's base) and where the wave's loads land
    unsigned voffA[IPK], voffB[NLB];
    {
#pragma unroll
        for (int h = 0; h < IPK; ++h) {               // the load's rows i = RPI h .. + RPI - 1 (its base points at row RPI h)
            const int il = lane / CPR, i = RPI * h + il, c = (lane % CPR) ^ ((i >> ISH) % CPR);
            voffA[h] = (unsigned)((VEC * c + (int64_t)il * g.rsA) * (int64_t)sizeof(T));
        }
#pragma unroll
        for (int j = 0; j < NLB; ++j) {
            const int u = NLB * wave + j;             // which KB of the B panel
            if (B_KC) {                               // 16 columns of 64 bytes
                const int col = 16 * u + (lane >> 2), ck = (lane & 3) ^ ((col >> 2) & 3);
                voffB[j] = (unsigned)(((int64_t)col * g.csB + VEC * ck) * (int64_t)sizeof(T));
            } else {                                  // whole k-rows of BN columns
                constexpr int LPR = BN / VEC;         // lanes per k-row
                const int kr = (64 / LPR) * u + lane / LPR, cc = lane % LPR;
                voffB[j] = (unsigned)(((int64_t)kr * g.rsB + VEC * cc) * (int64_t)sizeof(T));
            }
        }
    }
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) T *)lds;
    const unsigned landA = __builtin_amdgcn_readfirstlane(lds0 + wave * 4096);          // load 4 wave + j: + 1024 j
    const unsigned landB = __builtin_amdgcn_readfirstlane(lds0 + A_SIZE * (int)sizeof(T) + wave * (NLB * 1024));
    auto request = [&](int st, int64_t kb) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {                 // load t = 4 wave + j: k = t / IPK, rows from RPI (t % IPK)
            const int k = (4 * wave + j) / IPK, h = j % IPK;          // 4 wave is a multiple of IPK
            dma16(landA + st * (STAGE * (int)sizeof(T)) + j * 1024, A + (kb * BK + k) * g.csA + (int64_t)(RPI * h) * g.rsA, voffA[h]);
        }
#pragma unroll
        for (int j = 0; j < NLB; ++j)
            dma16(landB + st * (STAGE * (int)sizeof(T)) + j * 1024, B_KC ? B + kb * BK : B + kb * BK * g.rsB, voffB[j]);
    };

    typename MF::Acc acc[NBM][NBN];
#pragma unroll
    for (int a = 0; a < NBM; ++a)
#pragma unroll
        for (int c = 0; c < NBN; ++c)
#pragma unroll
            for (int r = 0; r < MF::NREG; ++r) acc[a][c][r] = S(0);

    const int rho0 = wave * (BM / 4), kl = lane / MI;
    Vec fa[2][NBM], fb[2][NBN];
    auto read_frags = [&](Vec (&xa)[NBM], Vec (&xb)[NBN], int st, int kg) __attribute__((always_inline)) {
        const T *As = lds + st * STAGE, *Bs = As + A_SIZE;
        const int k = kg * KF + kl * VEC;
#pragma unroll
        for (int a = 0; a < NBM; ++a) {
            const int rho = rho0 + a * MI + (lane % MI);
            const int i = rho % MB, b = rho / MB;
            const T *p = As + (i * CPR + ((b / VEC) ^ ((i >> ISH) % CPR))) * VEC + (b % VEC);
#pragma unroll
            for (int e = 0; e < VEC; ++e) xa[a][e] = p[(k + e) * (MB * PB)];
        }
        if constexpr (B_IL) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const ColVec v = *(const ColVec *)(Bs + (k + e) * BN + NBN * (lane % MI));
#pragma unroll
                for (int c = 0; c < NBN; ++c) xb[c][e] = v[c];
            }
            return;
        }
#pragma unroll
        for (int c = 0; c < NBN; ++c) {
            const int col = c * MI + (lane % MI);
            if (B_KC) {
                xb[c] = *(const Vec *)(Bs + (col * 4 + ((k / VEC) ^ ((col >> 2) & 3))) * VEC);
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) xb[c][e] = Bs[(k + e) * BN + col];
            }
        }
    };
    auto mfmas = [&](const Vec (&xa)[NBM], const Vec (&xb)[NBN]) __attribute__((always_inline)) {
        __builtin_amdgcn_s_setprio(2);
#pragma unroll
        for (int e = 0; e < STEPS; ++e)
#pragma unroll
            for (int a = 0; a < NBM; ++a)
#pragma unroll
                for (int c = 0; c < NBN; ++c) {
                    if (CT) MF::mma(acc[a][c], xa[a], xb[c], e);
                    else    MF::mma(acc[a][c], xb[c], xa[a], e);
                }
        __builtin_amdgcn_s_setprio(0);
    };

    request(0, 0);
    if (nkb > 1) {
        request(1, 1);
        dma_wait<4 + NLB>();         // panel 0 has landed; panel 1 may still be under way
    } else {
        dma_wait<0>();
    }
    __syncthreads();
    read_frags(fa[0], fb[0], 0, 0);
    if constexpr (KG == 2) {
        for (int64_t kb = 0; kb < nkb; ++kb) {
            const int st = (int)(kb & 1);
            read_frags(fa[1], fb[1], st, 1);
            mfmas(fa[0], fb[0]);
            __builtin_amdgcn_sched_barrier(0);
            dma_wait<0>();               // this wave's share of the next panel is in LDS
            __syncthreads();             // ... everybody's, and nobody reads this stage any more
            if (kb + 2 < nkb) request(st, kb + 2);
            __builtin_amdgcn_sched_barrier(0);
            if (kb + 1 < nkb) read_frags(fa[0], fb[0], st ^ 1, 0);
            mfmas(fa[1], fb[1]);
        }
    } else {
        // one fragment group per panel: panel kb's fragments are in set kb % 2 when its turn comes; the next
        // panel is waited for, published and read BEFORE this panel's MFMAs, which then cover those reads
        auto one = [&](int64_t kb, auto set_c) __attribute__((always_inline)) {
            constexpr int SET = decltype(set_c)::value;
            if (kb + 1 < nkb) {
                dma_wait<0>();
                __syncthreads();         // panel kb + 1 is in LDS, and everybody has finished reading panel kb's stage
                if (kb + 2 < nkb) request(SET, kb + 2);
                __builtin_amdgcn_sched_barrier(0);
                read_frags(fa[SET ^ 1], fb[SET ^ 1], SET ^ 1, 0);
            }
            mfmas(fa[SET], fb[SET]);
        };
        for (int64_t kb = 0; kb < nkb; kb += 2) {
            one(kb, std::integral_constant<int, 0>());
            if (kb + 1 < nkb) one(kb + 1, std::integral_constant<int, 1>());
        }
    }

    // epilogue (whole bricks only): as in the kernel above
    const S alpha = (S)g.alpha, beta = (S)g.beta;
    auto store_tile = [&](auto beta_c) __attribute__((always_inline)) {
        constexpr bool BETA = decltype(beta_c)::value;
        if (CT) {
#pragma unroll
            for (int c = 0; c < NBN; ++c) {
                T *Cc = (T *)g.C + o1.c + (j0 + c * MI + (lane % MI));
#pragma unroll
                for (int a = 0; a < NBM; ++a)
#pragma unroll
                    for (int r = 0; r < MF::NREG; ++r) {
                        const int rho = rho0 + a * MI + MF::row_lane(lane) + MF::row_reg(r);
                        T *dst = Cc + (bb + rho / MB) * g.bsC[0] + (i0 + rho % MB) * g.ldc;
                        S v = alpha * acc[a][c][r];
                        if (BETA) v += beta * *dst;
                        *dst = v;
                    }
            }
            return;
        }
#pragma unroll
        for (int a = 0; a < NBM; ++a) {
            const int rho = rho0 + a * MI + (lane % MI);
            T *Cb = (T *)g.C + (bb + rho / MB) * g.bsC[0] + o1.c + (i0 + rho % MB);
#pragma unroll
            for (int c = 0; c < NBN; ++c) {
#pragma unroll
                for (int r = 0; r < MF::NREG; ++r) {
                    const int idx = MF::row_lane(lane) + MF::row_reg(r);        // index of the column inside its MFMA block
                    T *dst = Cb + (j0 + (B_IL ? NBN * idx + c : c * MI + idx)) * g.ldc;
                    S v = alpha * acc[a][c][r];
                    if (BETA) v += beta * *dst;
                    *dst = v;
                }
            }
        }
    };
    if (beta == S(0)) store_tile(std::false_type());
    else              store_tile(std::true_type());
}

// the direct-to-LDS member takes whole bricks (64 bytes of k per panel) whose every load is 16-byte aligned and
// whose lane offsets fit 32 bits; vec: elements per 16 bytes
bool dma_applies(const SbArgs &a, int vec)
{
    const int bk = 16 * vec / 4;
    if (a.batch0 % 16 || a.m % 16 || a.n % 64 || a.k % bk || a.k < bk) return false;
    auto al = [vec](int64_t v) { return v % vec == 0; };
    const int64_t ldB = a.rsB == 1 ? a.csB : a.rsB;
    if (((uintptr_t)a.A | (uintptr_t)a.B) % 16) return false;
    if (!al(a.rsA) || !al(a.csA) || !al(ldB) || !al(a.bsA[1]) || !al(a.bsB[1])) return false;
    for (int x = 0; x < a.nx; ++x)
        if (!al(a.xsA[x]) || !al(a.xsB[x])) return false;
    // lane offsets are 32-bit byte offsets: up to 15 rows of A, up to 127 columns (or 15 k-rows) of B
    return a.rsA > 0 && a.rsA < ((int64_t)1 << 24) && a.csA > 0 && ldB > 0 && ldB < ((int64_t)1 << 22);
}

template <typename MF, bool CT, int BN>
hipError_t launch_dma(const SbArgs &a, hipStream_t stream)
{
    const int64_t tiles_b = a.batch0 / 16, tiles_i = a.m / 16, tiles_n = a.n / BN;
    const int64_t total = tiles_b * tiles_i * tiles_n * a.batch1;
    if (total <= 0) return hipSuccess;
    if (total > sb_max_grid_x(256)) return hipErrorInvalidConfiguration;
    dim3 grid((unsigned)total), block(256);
    if (a.rsB == 1) hipLaunchKernelGGL((sbgemm_mfma_exa_dma_kernel<MF, true, CT, BN>), grid, block, 0, stream, a, (int)tiles_b, (int)tiles_i, (int)tiles_n);
    else            hipLaunchKernelGGL((sbgemm_mfma_exa_dma_kernel<MF, false, CT, BN>), grid, block, 0, stream, a, (int)tiles_b, (int)tiles_i, (int)tiles_n);
    return hipGetLastError();
}

template <typename MF, bool CT, int PB, int MB, int BN, int BK>
hipError_t launch(const SbArgs &a, hipStream_t stream)
{
    const int64_t tiles_b = (a.batch0 + PB - 1) / PB, tiles_i = (a.m + MB - 1) / MB, tiles_n = (a.n + BN - 1) / BN;
    const int64_t total = tiles_b * tiles_i * tiles_n * a.batch1;
    if (total <= 0) return hipSuccess;
    if (total > sb_max_grid_x(ET)) return hipErrorInvalidConfiguration;           // sb_mfma_exa_supports keeps such problems away
    // 16-byte vector loads need no alignment beyond the element's: the hardware reads them anywhere
    const int vec_a = 1, vec_b = 1;
    dim3 grid((unsigned)total), block(ET);
    if (a.rsB == 1) hipLaunchKernelGGL((sbgemm_mfma_exa_kernel<MF, true, CT, PB, MB, BN, BK>), grid, block, 0, stream, a, (int)tiles_b, (int)tiles_i, (int)tiles_n, vec_a, vec_b);
    else            hipLaunchKernelGGL((sbgemm_mfma_exa_kernel<MF, false, CT, PB, MB, BN, BK>), grid, block, 0, stream, a, (int)tiles_b, (int)tiles_i, (int)tiles_n, vec_a, vec_b);
    return hipGetLastError();
}

// first-operand form: A strided in rows and columns with level-0 batch stride 1, B a plain N/T matrix that
// does not move with level 0
bool first_form(const SbArgs &a)
{
    if (a.k <= 0 || a.batch0 < 8) return false;
    if (a.bsA[0] != 1 || a.rsA == 1 || a.csA == 1) return false;
    if (a.bsB[0] != 0) return false;
    if (a.rsB != 1 && a.csB != 1) return false;
    // one workgroup per tile of at least 16 batches x 16 rows x 32 columns, in a one-dimensional grid
    const int64_t tiles = ((a.batch0 + 15) / 16) * ((a.m + 15) / 16) * ((a.n + 31) / 32) * a.batch1;
    if (tiles > sb_max_grid_x(ET)) return false;
    return a.m >= 8 && a.n >= 16;
}

// the transposed problem C^T = op(B)^T op(A)^T: operands and their batch strides trade places, rows and
// columns of each trade places; C itself is untouched (the kernel writes its tile transposed)
SbArgs transposed(const SbArgs &a)
{
    SbArgs t = a;
    t.A = a.B;  t.B = a.A;
    t.m = a.n;  t.n = a.m;
    t.rsA = a.csB;  t.csA = a.rsB;
    t.rsB = a.csA;  t.csB = a.rsA;
    for (int l = 0; l < 2; ++l) { t.bsA[l] = a.bsB[l];  t.bsB[l] = a.bsA[l]; }
    for (int x = 0; x < SB_MAX_BATCH_LEVELS - 2; ++x) { t.xsA[x] = a.xsB[x];  t.xsB[x] = a.xsA[x]; }
    return t;
}

}  // namespace

// One operand is "extended" (level-0 batch stride 1, rows and columns both strided), the other is a plain
// N/T matrix that does not move with batch level 0, C_b are ordinary column-major matrices.
bool sb_mfma_exa_supports(sb_dtype dt, const SbArgs &a)
{
    return first_form(a) || first_form(transposed(a));
}

// Tiles: 16 batches x 16 rows x 64 columns and 16 k per panel (fp64: 32 columns, 8 k; bf16: 32 k).  A problem
// that makes fewer than 128 such tiles (64^4: 16) would leave most of the chip idle behind long chains of
// dependent MFMAs (128 per wave at 64^4), so fp32 and fp64 then take tiles of a quarter the size: 16 batches x
// 8 rows x 32 columns (fp64: 4 rows x 16 columns), one MFMA block per wave.
template <bool CT>
static hipError_t launch_form(sb_dtype dt, const SbArgs &a, hipStream_t stream)
{
    const int64_t bn = dt == SB_F64 ? 32 : 64;
    const bool few = ((a.batch0 + 15) / 16) * ((a.m + 15) / 16) * ((a.n + bn - 1) / bn) * a.batch1 < 128;
    if (dt == SB_F32 && !few && dma_applies(a, 4)) {
        sb_note_member(SB_MEMBER_MFMA_EX_DMA);
        // 128-column tiles when they still make a full round of workgroups (two per compute unit)
        const bool wide = a.n % 128 == 0 && (a.batch0 / 16) * (a.m / 16) * (a.n / 128) * a.batch1 >= 512;
        return wide ? launch_dma<ExF32, CT, 128>(a, stream) : launch_dma<ExF32, CT, 64>(a, stream);
    }
    if (dt == SB_F64 && !few && dma_applies(a, 2)) {
        sb_note_member(SB_MEMBER_MFMA_EX_DMA);
        return launch_dma<ExF64, CT, 64>(a, stream);
    }
    sb_note_member(few && dt != SB_BF16 ? SB_MEMBER_MFMA_EX_SMALL : SB_MEMBER_MFMA_EX_BRICK);
    if (dt == SB_F32) return few ? launch<ExF32, CT, 16, 8, 32, 16>(a, stream) : launch<ExF32, CT, 16, 16, 64, 16>(a, stream);
    if (dt == SB_F64) return few ? launch<ExF64, CT, 16, 4, 16, 8>(a, stream) : launch<ExF64, CT, 16, 16, 32, 8>(a, stream);
    if (dt == SB_BF16) return launch<ExBf16, CT, 16, 16, 64, 32>(a, stream);
    return hipErrorInvalidValue;
}

hipError_t sb_launch_mfma_exa(sb_dtype dt, const SbArgs &a, hipStream_t stream)
{
    if (first_form(a)) return launch_form<false>(dt, a, stream);
    const SbArgs t = transposed(a);
    if (!first_form(t)) return hipErrorInvalidValue;
    return launch_form<true>(dt, t, stream);
}
