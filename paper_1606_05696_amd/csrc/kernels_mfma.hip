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

#include <atomic>
#include <type_traits>

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef double f64x4 __attribute__((ext_vector_type(4)));

// Instruction traits.  MI: block edge; the 64/MI lane groups each hold VEC consecutive k, so one
// fragment read covers KGROUP = (64/MI)*VEC values of k and feeds VEC consecutive MFMAs.

// v_mfma_f32_32x32x2_f32: operands hold X[l%32][k = l/32]; result slot r of lane l is
// D[8*(r/4) + 4*(l/32) + r%4][l%32] (a lane part plus a register part).
struct MfmaF32x32 {
    typedef float T;
    static constexpr int MI = 32, VEC = 4, NREG = 16, KGROUP = 8;
    typedef f32x16 Acc;
    typedef float Vec __attribute__((ext_vector_type(4)));
    typedef float VecU __attribute__((ext_vector_type(4), aligned(4)));       // a vector at any element address
    static __device__ __forceinline__ void mma(Acc &c, float first, float second)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(first, second, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int result_row_lane(int lane) { return 4 * (lane >> 5); }
    static constexpr int result_row_reg(int r) { return 8 * (r >> 2) + (r & 3); }
};

// v_mfma_f64_16x16x4_f64: operands hold X[l%16][k = l/16]; result slot r of lane l is D[l/16 + 4*r][l%16].
struct MfmaF64x16 {
    typedef double T;
    static constexpr int MI = 16, VEC = 2, NREG = 4, KGROUP = 8;
    typedef f64x4 Acc;
    typedef double Vec __attribute__((ext_vector_type(2)));
    typedef double VecU __attribute__((ext_vector_type(2), aligned(8)));
    static __device__ __forceinline__ void mma(Acc &c, double first, double second)
    {
        c = __builtin_amdgcn_mfma_f64_16x16x4f64(first, second, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int result_row_lane(int lane) { return lane >> 4; }
    static constexpr int result_row_reg(int r) { return 4 * r; }
};

constexpr int NXCD = 8;

// Stage one BK-deep panel (ROWS rows of the operand) from global memory into registers.
// KC: the panel is stored [row][k] with k contiguous in memory (row stride `ld`);
// otherwise rows are contiguous and k strides by `ld`.
template <typename MF, bool KC, int ROWS, int BK, int NT>
struct Panel {
    typedef typename MF::T T;
    typedef typename MF::Vec Vec;
    typedef typename MF::VecU VecU;      // global loads: gfx950 reads a 16-byte vector at any element-aligned address
    static constexpr int VEC = MF::VEC;
    static constexpr int NVEC = ROWS * BK / VEC / NT;                  // 16-byte vectors per lane
    // k-contiguous panels are stored unpadded, the 16-byte chunk c of row r at chunk c ^ f(r) with
    // f(r) = (r / rows-per-256-bytes) mod chunks-per-row: sixteen lanes that store consecutive chunks
    // cover 256 contiguous bytes, sixteen lanes that read the same chunk of consecutive rows (an
    // MFMA fragment) hit sixteen different groups of four banks, so neither conflicts.  (Padded
    // rows keep the reads apart but let a store wrap onto the banks of the row three above: a third
    // of the LDS cycles of the 128 x 128 kernels were bank conflicts.)  Row-contiguous panels keep
    // the padding.
    static constexpr int CPR = BK / VEC;                               // chunks per row
    static_assert(!KC || (CPR <= 16 && (CPR & (CPR - 1)) == 0), "chunks per row: a power of two up to 16");
    static constexpr int LDS_LD = KC ? BK : ROWS + VEC;
    static constexpr int LDS_SIZE = (KC ? ROWS : BK) * LDS_LD;
    static __device__ __forceinline__ int swizzled(int row, int k)     // k a multiple of VEC
    {
        return ((k / VEC) ^ ((row / (16 / CPR)) & (CPR - 1))) * VEC;
    }
    static_assert(ROWS * BK % (VEC * NT) == 0, "panel must split evenly over the lanes");

    static __device__ __forceinline__ void coords(int f, int &row, int &k)
    {
        if (KC) { row = f / (BK / VEC); k = (f % (BK / VEC)) * VEC; }
        else    { k = f / (ROWS / VEC); row = (f % (ROWS / VEC)) * VEC; }
    }

    // GUARD = 0: the whole panel lies inside the matrix and every vector is 16-byte aligned.
    // GUARD = 1: edge tile whose edges fall between vectors (aligned operands, the extent along the
    //            contiguous dimension a multiple of the vector length): every lane still issues its
    //            vector load, from a safe address when its vector lies outside, and zeroes it then;
    //            no branch, so the loads stay countable and pipelined exactly as in an interior tile.
    // GUARD = 2: rows_left / k_left say how much of the panel is inside, element by element (odd
    //            extents, unaligned operands).
    template <int GUARD>
    static __device__ __forceinline__ void load(Vec (&v)[NVEC], const T *p, int64_t ld, int64_t rows_left, int64_t k_left, bool vec_ok)
    {
#pragma unroll
        for (int q = 0; q < NVEC; ++q) {
            int row, k;
            coords((int)threadIdx.x + NT * q, row, k);
            const T *src = KC ? p + (int64_t)row * ld + k : p + (int64_t)k * ld + row;
            if (GUARD == 0) {
                v[q] = *(const VecU *)src;
                continue;
            }
            if (GUARD == 1) {          // the vector is zeroed when it goes to LDS: masking it here would wait for the load
                const bool in = row < rows_left && k < k_left;
                v[q] = *(const VecU *)(in ? src : p);
                continue;
            }
            const bool inside = KC ? (row < rows_left && k + VEC <= k_left) : (row + VEC <= rows_left && k < k_left);
            if (vec_ok && inside) {
                v[q] = *(const VecU *)src;
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const bool ok = KC ? (row < rows_left && k + e < k_left) : (row + e < rows_left && k < k_left);
                    v[q][e] = ok ? src[e] : T(0);
                }
            }
        }
    }

    // MASK: the panel was loaded with GUARD = 1; vectors outside the matrix become zeros here
    template <bool MASK = false>
    static __device__ __forceinline__ void store(T *lds, const Vec (&v)[NVEC], int64_t rows_left = 0, int64_t k_left = 0)
    {
#pragma unroll
        for (int q = 0; q < NVEC; ++q) {
            int row, k;
            coords((int)threadIdx.x + NT * q, row, k);
            T *dst = KC ? lds + row * LDS_LD + swizzled(row, k) : lds + k * LDS_LD + row;
            *(Vec *)dst = (!MASK || (row < rows_left && k < k_left)) ? v[q] : Vec(T(0));
        }
    }

    // Fragment of the MFMA block whose first row is row0, for k-group kg: VEC consecutive MFMA steps.
    static __device__ __forceinline__ void fragment(T (&frag)[VEC], const T *lds, int row0, int kg, int lane)
    {
        constexpr int MI = MF::MI;
        const int row = row0 + (lane % MI);
        const int k = kg * MF::KGROUP + (lane / MI) * VEC;
        if (KC) {
            Vec v = *(const Vec *)(lds + row * LDS_LD + swizzled(row, k));
#pragma unroll
            for (int e = 0; e < VEC; ++e) frag[e] = v[e];
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) frag[e] = lds[(k + e) * LDS_LD + row];
        }
    }
};

// Tile configuration: each wave owns WM x WN of C; WAVES_M x WAVES_N waves form the workgroup tile.
template <typename MFT, bool A_KC, bool B_KC, int BK, int WM, int WN, int WAVES_M, int WAVES_N, int GD = 2>
struct Config {
    static constexpr int GDIST = GD;      // how many panels ahead the global loads run (1 or 2)
    static constexpr int BM = WM * WAVES_M, BN = WN * WAVES_N, BKC = BK;
    static constexpr int NT = 64 * WAVES_M * WAVES_N;
    typedef MFT MF;
    static_assert((BK / MF::KGROUP) % 2 == 0, "the fragment double buffer needs an even number of k-groups per panel");
    typedef Panel<MF, A_KC, BM, BK, NT> PA;
    typedef Panel<MF, B_KC, BN, BK, NT> PB;
    static constexpr int NBM = WM / MF::MI, NBN = WN / MF::MI;         // MFMA blocks per wave tile
};

// The k loop of one tile, software-pipelined at two levels:
//   - global -> registers: the panel for block kb+2 is requested while block kb is being multiplied
//     (two staging register sets), so a full iteration of MFMAs covers the memory latency;
//   - LDS -> registers: the fragments of the next k-group are read while the current group's
//     MFMAs run (two fragment register sets).  The hand-over to the next block (LDS store of the
//     staged panel, barrier, first fragment read of the new block) is placed BEFORE the last
//     k-group's MFMAs of the current block, which then hide its latency.
// GA / GB select, per operand, bounds-checked scalar loads (odd extents, unaligned operands),
// masked vector loads (edge tiles whose edges fall between vectors) or plain 16-byte vector loads
// (interior tiles, branch-free): a ragged or unaligned operand does not slow the other one down.
template <typename CF, typename T, int GA, int GB>
__device__ __forceinline__ void k_loop(typename CF::MF::Acc (&acc)[CF::NBM][CF::NBN], T (*As)[CF::PA::LDS_SIZE], T (*Bs)[CF::PB::LDS_SIZE],
                                        const T *A, const T *B, int64_t ldA, int64_t ldB, int64_t kstepA, int64_t kstepB,
                                        int64_t m_left, int64_t n_left, int64_t K, bool vec_a, bool vec_b, int wm, int wn, int lane, int BKc)
{
    typedef typename CF::MF MF;
    typedef typename CF::PA PA;
    typedef typename CF::PB PB;
    constexpr int MI = MF::MI, VEC = MF::VEC, BK = CF::BKC, KG = BK / MF::KGROUP;
    (void)BKc;
    constexpr int GD = CF::GDIST;
    typename PA::Vec ra[GD][PA::NVEC];
    typename PB::Vec rb[GD][PB::NVEC];
    T fa[2][CF::NBM][VEC], fb[2][CF::NBN][VEC];
    const int64_t nkb = (K + BK - 1) / BK;

    auto read_frags = [&](auto set, auto buf, int kg) {
#pragma unroll
        for (int a = 0; a < CF::NBM; ++a) PA::fragment(fa[set][a], As[buf], wm + a * MI, kg, lane);
#pragma unroll
        for (int c = 0; c < CF::NBN; ++c) PB::fragment(fb[set][c], Bs[buf], wn + c * MI, kg, lane);
    };
    auto gload = [&](auto set, int64_t kb) {
        const int64_t k0 = kb * BK;
        PA::template load<GA>(ra[set], A + k0 * kstepA, ldA, m_left, K - k0, vec_a);
        PB::template load<GB>(rb[set], B + k0 * kstepB, ldB, n_left, K - k0, vec_b);
    };
    // one k block; CUR (= kb & 1) is a compile-time constant so that every register array is
    // indexed statically.  STEADY = true is the steady state (block kb+2 exists): the prefetch
    // and the hand-over are unconditional, which lets the compiler count outstanding loads exactly
    // and wait only for the older staging set.
    auto block = [&](auto cur_c, auto steady_c, int64_t kb) {
        constexpr int CUR = decltype(cur_c)::value;
        constexpr bool STEADY = decltype(steady_c)::value;
        if (STEADY || kb + GD < nkb) gload(std::integral_constant<int, (GD == 2 ? CUR : 0)>(), kb + GD);   // this staging set was consumed one block ago
#pragma unroll
        for (int kg = 0; kg < KG; ++kg) {
            const int fs = kg & 1;
            const bool hand_over = STEADY || kb + 1 < nkb;
            if (kg + 1 < KG) {
                if (fs == 0) read_frags(std::integral_constant<int, 1>(), std::integral_constant<int, CUR>(), kg + 1);
                else         read_frags(std::integral_constant<int, 0>(), std::integral_constant<int, CUR>(), kg + 1);
            } else if (hand_over) {
                // the staged panel went to LDS in the middle of the previous cluster, so this
                // barrier finds the stores complete and costs only the skew between the waves
                __syncthreads();
                read_frags(std::integral_constant<int, 0>(), std::integral_constant<int, CUR ^ 1>(), 0);
            }
            // Raised priority inside the MFMA cluster: the wave that enters first keeps the matrix
            // core until its cluster ends instead of sharing it turn by turn, so the co-resident
            // waves drift out of phase and one wave's memory phase hides under another's MFMAs.
            __builtin_amdgcn_s_setprio(2);
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                if (e == VEC / 2 && kg == KG - 2 && hand_over) {
                    // LDS store of the next block's panel (requested one block ago) between two
                    // halves of a cluster: the matrix core keeps running under it
                    __builtin_amdgcn_sched_barrier(0);
                    PA::template store<GA == 1>(As[CUR ^ 1], ra[GD == 2 ? (CUR ^ 1) : 0], m_left, K - (kb + 1) * BK);
                    PB::template store<GB == 1>(Bs[CUR ^ 1], rb[GD == 2 ? (CUR ^ 1) : 0], n_left, K - (kb + 1) * BK);
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int a = 0; a < CF::NBM; ++a)
#pragma unroll
                    for (int c = 0; c < CF::NBN; ++c) MF::mma(acc[a][c], fb[fs][c][e], fa[fs][a][e]);   // C^T = B^T A^T
            }
            __builtin_amdgcn_s_setprio(0);
        }
    };
    typedef std::integral_constant<int, 0> I0;
    typedef std::integral_constant<int, 1> I1;

    gload(I0(), 0);
    if (GD == 2 && nkb > 1) gload(std::integral_constant<int, GD - 1>(), 1);
    PA::template store<GA == 1>(As[0], ra[0], m_left, K);
    PB::template store<GB == 1>(Bs[0], rb[0], n_left, K);
    __syncthreads();
    read_frags(I0(), I0(), 0);
    int64_t kb = 0;
    for (; kb + 1 + GD < nkb; kb += 2) {               // steady state, two blocks per trip
        block(I0(), std::true_type(), kb);
        block(I1(), std::true_type(), kb + 1);
    }
    for (; kb < nkb; kb += 2) {                        // last one to three blocks
        block(I0(), std::false_type(), kb);
        if (kb + 1 < nkb) block(I1(), std::false_type(), kb + 1);
    }
}

// Second launch bound: the 4-wave configurations must leave room for two workgroups per compute unit
// (256 registers per lane); some operand orientations would otherwise take 290 and run alone.
template <typename MFT, bool A_KC, bool B_KC, int BK, int WM, int WN, int WAVES_M, int WAVES_N, int GD>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N, WAVES_M * WAVES_N <= 4 ? 2 : 1) void sbgemm_mfma_kernel(SbArgs g, int tiles_m, int tiles_n, int vec_ok)
{
    typedef Config<MFT, A_KC, B_KC, BK, WM, WN, WAVES_M, WAVES_N, GD> CF;
    typedef typename CF::MF MF;
    typedef typename MF::T T;
    constexpr int MI = MF::MI, BM = CF::BM, BN = CF::BN;
    __shared__ __attribute__((aligned(16))) T As[2][CF::PA::LDS_SIZE];
    __shared__ __attribute__((aligned(16))) T Bs[2][CF::PB::LDS_SIZE];

    const int64_t ldA = A_KC ? g.rsA : g.csA;
    const int64_t ldB = B_KC ? g.csB : g.rsB;
    const int64_t kstepA = A_KC ? 1 : g.csA;
    const int64_t kstepB = B_KC ? 1 : g.rsB;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave % WAVES_M) * WM, wn = (wave / WAVES_M) * WN;
    const T alpha = (T)g.alpha, beta = (T)g.beta;

    // Persistent workgroups: the grid holds as many workgroups as the chip can keep resident and
    // each walks over several tiles.  The stores of one tile are only queued, not waited for, so
    // they drain while the next tile's panels are fetched and multiplied; with one tile per
    // workgroup all workgroups would reach their store phase together and the matrix cores
    // would idle during every such burst.
    // XCD-aware order: hardware hands consecutive workgroup ids to the 8 XCDs in turn, so workgroup
    // w sits on XCD w % 8; each XCD gets one contiguous range of tiles (the tiles of one batch
    // share B_p in its L2) and its workgroups take them round-robin.
    const int64_t tiles = (int64_t)tiles_m * tiles_n;
    const int64_t total = tiles * g.batch0 * g.batch1;
    const int64_t nslots = (int64_t)gridDim.x / NXCD;              // the launcher makes gridDim.x a multiple of 8
    const int64_t xcd = blockIdx.x % NXCD, slot = blockIdx.x / NXCD;
    const int64_t q8 = total / NXCD, r8 = total % NXCD;
    const int64_t first = xcd * q8 + (xcd < r8 ? xcd : r8);
    const int64_t last = first + q8 + (xcd < r8 ? 1 : 0);

    for (int64_t logical = first + slot; logical < last; logical += nslots) {
        const int64_t b = logical / tiles;
        const int tile = (int)(logical - b * tiles);
        const int64_t b1 = b / g.batch0, b0 = b - b1 * g.batch0;
        const SbOff3 o1 = sb_level1(g, b1);
        const int tm = tile % tiles_m, tn = tile / tiles_m;
        const int64_t i0 = (int64_t)tm * BM, j0 = (int64_t)tn * BN;

        // op(A)(i,l) = A[i*rsA + l*csA]: with k contiguous the row stride is rsA, else the k stride is csA
        const T *A = (const T *)g.A + b0 * g.bsA[0] + o1.a + i0 * g.rsA;
        const T *B = (const T *)g.B + b0 * g.bsB[0] + o1.b + j0 * g.csB;
        T *C = (T *)g.C + b0 * g.bsC[0] + o1.c;
        const int64_t m_left = g.m - i0, n_left = g.n - j0;

        typename MF::Acc acc[CF::NBM][CF::NBN];
#pragma unroll
        for (int a = 0; a < CF::NBM; ++a)
#pragma unroll
            for (int c = 0; c < CF::NBN; ++c)
#pragma unroll
                for (int r = 0; r < MF::NREG; ++r) acc[a][c][r] = T(0);

        // workgroup-uniform choices.  Interior tile with aligned operands: branch-free loop.
        // Otherwise, per operand: if its panels' edges fall between 16-byte vectors (aligned, and the
        // extent along its contiguous dimension whole vectors or not cut by this tile), masked
        // unconditional vector loads; else element-wise guards.
        const bool vec_a = vec_ok & 1, vec_b = vec_ok & 2;
        const bool interior = vec_a && vec_b && m_left >= BM && n_left >= BN && (g.k % BK == 0);
        const bool mask_a = vec_a && (A_KC ? g.k % MF::VEC == 0 : (m_left >= BM || g.m % MF::VEC == 0));
        const bool mask_b = vec_b && (B_KC ? g.k % MF::VEC == 0 : (n_left >= BN || g.n % MF::VEC == 0));
#define K_LOOP(GA, GB) k_loop<CF, T, GA, GB>(acc, As, Bs, A, B, ldA, ldB, kstepA, kstepB, m_left, n_left, g.k, vec_a, vec_b, wm, wn, lane, BK)
        if (interior)               K_LOOP(0, 0);
        else if (mask_a && mask_b)  K_LOOP(1, 1);
        else if (mask_a)            K_LOOP(1, 2);
        else if (mask_b)            K_LOOP(2, 1);
        else                        K_LOOP(2, 2);
#undef K_LOOP

        // epilogue: lane = row of C within the block, result slot = column.  The four variants
        // (edge tile or not, beta or not) are chosen by workgroup-uniform branches so that the
        // common one is a straight run of stores.
        auto store_tile = [&](auto guard_c, auto beta_c) {
            constexpr bool GUARD = decltype(guard_c)::value, BETA = decltype(beta_c)::value;
#pragma unroll
            for (int a = 0; a < CF::NBM; ++a) {
                const int64_t i = i0 + wm + a * MI + (lane % MI);
                if (GUARD && i >= g.m) continue;
#pragma unroll
                for (int c = 0; c < CF::NBN; ++c) {
                    const int64_t jl = j0 + wn + c * MI + MF::result_row_lane(lane);
                    T *col = C + i + jl * g.ldc;
#pragma unroll
                    for (int r = 0; r < MF::NREG; ++r) {
                        if (GUARD && jl + MF::result_row_reg(r) >= g.n) continue;
                        T *dst = col + MF::result_row_reg(r) * g.ldc;
                        T v = alpha * acc[a][c][r];
                        if (BETA) v += beta * *dst;
                        *dst = v;
                    }
                }
            }
        };
        const bool edge = m_left < BM || n_left < BN;
        if (!edge) {
            if (beta == T(0)) store_tile(std::false_type(), std::false_type());
            else              store_tile(std::false_type(), std::true_type());
        } else {
            if (beta == T(0)) store_tile(std::true_type(), std::false_type());
            else              store_tile(std::true_type(), std::true_type());
        }
        __syncthreads();      // every wave is done with the LDS panels before the next tile refills them
    }
}

// Streaming variant for problems made of whole tiles (m, n multiples of the tile, k a multiple of
// 2*BK and at least 4*BK, aligned operands): the panel stream never drains at a tile boundary.
// While the last k blocks of a tile are multiplied, the first panels of the workgroup's NEXT tile
// are already being fetched and handed to LDS, so a new tile starts multiplying as soon as the old
// tile's results are queued for storing; no memory latency is exposed between tiles.
//   - The loads of the next tile's third panel are issued BEFORE the stores of the finished tile:
//     gfx9 counts loads and stores in one in-order counter, so a wait for a load issued after the
//     stores would also wait for every store.  With this order the first waits that include the
//     stores come two k blocks into the new tile.
//   - The body of a tile exists twice (first tile after the explicit priming, all later tiles in
//     a loop), and beta != 0 is a kernel of its own: where two paths with different numbers of
//     outstanding memory operations meet, the compiler must wait for the smaller count, which
//     here would mean "until the previous tile's stores have drained".
//   - The last tile of a workgroup prefetches its own first panels again (in bounds, never used).
template <typename MFT, bool A_KC, bool B_KC, bool BETA, int BK, int WM, int WN, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void sbgemm_mfma_stream_kernel(SbArgs g, int tiles_m, int tiles_n)
{
    typedef Config<MFT, A_KC, B_KC, BK, WM, WN, WAVES_M, WAVES_N, 2> CF;
    typedef typename CF::MF MF;
    typedef typename MF::T T;
    typedef typename CF::PA PA;
    typedef typename CF::PB PB;
    constexpr int MI = MF::MI, VEC = MF::VEC, BM = CF::BM, BN = CF::BN, KG = BK / MF::KGROUP;
    __shared__ __attribute__((aligned(16))) T As[2][PA::LDS_SIZE];
    __shared__ __attribute__((aligned(16))) T Bs[2][PB::LDS_SIZE];

    const int64_t ldA = A_KC ? g.rsA : g.csA;
    const int64_t ldB = B_KC ? g.csB : g.rsB;
    const int64_t stepA = (A_KC ? 1 : g.csA) * BK, stepB = (B_KC ? 1 : g.rsB) * BK;      // one panel along k
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave % WAVES_M) * WM, wn = (wave / WAVES_M) * WN;
    const T alpha = (T)g.alpha, beta = (T)g.beta;
    const int64_t nkb = g.k / BK;

    // same persistent, XCD-aware schedule as sbgemm_mfma_kernel
    const int64_t tiles = (int64_t)tiles_m * tiles_n;
    const int64_t total = tiles * g.batch0 * g.batch1;
    const int64_t nslots = (int64_t)gridDim.x / NXCD;
    const int64_t xcd = blockIdx.x % NXCD, slot = blockIdx.x / NXCD;
    const int64_t q8 = total / NXCD, r8 = total % NXCD;
    const int64_t first = xcd * q8 + (xcd < r8 ? xcd : r8);
    const int64_t last = first + q8 + (xcd < r8 ? 1 : 0);
    int64_t logical = first + slot;
    if (logical >= last) return;

    typename PA::Vec ra[2][PA::NVEC];
    typename PB::Vec rb[2][PB::NVEC];
    T fa[2][CF::NBM][VEC], fb[2][CF::NBN][VEC];
    typename MF::Acc acc[CF::NBM][CF::NBN];

    // tile number -> operand pointers.  The walk over the tiles advances (batch, tile) by addition;
    // 64-bit divisions at every tile boundary would sit right where the matrix cores wait.
    struct Loc { const T *A, *B; T *C; };
    auto locate = [&](int64_t b, int tile) {
        int64_t b0 = b, b1 = 0;
        if (g.batch1 != 1) { b1 = b / g.batch0; b0 = b - b1 * g.batch0; }
        const SbOff3 o1 = sb_level1(g, b1);
        const unsigned tn = (unsigned)tile / (unsigned)tiles_m, tm = (unsigned)tile - tn * (unsigned)tiles_m;
        const int64_t i0 = (int64_t)tm * BM, j0 = (int64_t)tn * BN;
        Loc l;
        l.A = (const T *)g.A + b0 * g.bsA[0] + o1.a + i0 * g.rsA;
        l.B = (const T *)g.B + b0 * g.bsB[0] + o1.b + j0 * g.csB;
        l.C = (T *)g.C + b0 * g.bsC[0] + o1.c + i0 + j0 * g.ldc;
        return l;
    };
    int64_t b = logical / tiles;
    int tile = (int)(logical - b * tiles);
    const int64_t dq = nslots / tiles;
    const int dr = (int)(nslots - dq * tiles);
    auto gload = [&](auto set, const T *pa, const T *pb) {
        PA::template load<false>(ra[set], pa, ldA, 0, 0, true);
        PB::template load<false>(rb[set], pb, ldB, 0, 0, true);
    };
    auto read_frags = [&](auto set, auto buf, int kg) {
#pragma unroll
        for (int a = 0; a < CF::NBM; ++a) PA::fragment(fa[set][a], As[buf], wm + a * MI, kg, lane);
#pragma unroll
        for (int c = 0; c < CF::NBN; ++c) PB::fragment(fb[set][c], Bs[buf], wn + c * MI, kg, lane);
    };
    typedef std::integral_constant<int, 0> I0;
    typedef std::integral_constant<int, 1> I1;
    // One k block of the stream (CUR = parity of the block): optionally request the panel two
    // blocks ahead into the staging set this block's panel came from, multiply, and hand the next
    // block's panel to LDS in the middle of the second-to-last MFMA cluster.
    auto block = [&](auto cur_c, auto load_c, const T *pa, const T *pb) {
        constexpr int CUR = decltype(cur_c)::value;
        if (decltype(load_c)::value) gload(std::integral_constant<int, CUR>(), pa, pb);
#pragma unroll
        for (int kg = 0; kg < KG; ++kg) {
            const int fs = kg & 1;
            if (kg + 1 < KG) {
                if (fs == 0) read_frags(I1(), std::integral_constant<int, CUR>(), kg + 1);
                else         read_frags(I0(), std::integral_constant<int, CUR>(), kg + 1);
            } else {
                __syncthreads();
                read_frags(I0(), std::integral_constant<int, CUR ^ 1>(), 0);
            }
            __builtin_amdgcn_s_setprio(2);
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                if (e == VEC / 2 && kg == KG - 2) {
                    __builtin_amdgcn_sched_barrier(0);
                    PA::store(As[CUR ^ 1], ra[CUR ^ 1]);
                    PB::store(Bs[CUR ^ 1], rb[CUR ^ 1]);
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int a = 0; a < CF::NBM; ++a)
#pragma unroll
                    for (int c = 0; c < CF::NBN; ++c) MF::mma(acc[a][c], fb[fs][c][e], fa[fs][a][e]);   // C^T = B^T A^T
            }
            __builtin_amdgcn_s_setprio(0);
        }
    };
    // One tile.  On entry its panel 0 is in LDS buffer 0 with the first fragments read, panel 1 is
    // in staging set 1 (in flight), panel 2 in staging set 0 (in flight).
    auto run_tile = [&](const Loc &cur, const Loc &nxt) {
        const T *A = cur.A, *B = cur.B, *An = nxt.A, *Bn = nxt.B;
        T *C = cur.C;
#pragma unroll
        for (int a = 0; a < CF::NBM; ++a)
#pragma unroll
            for (int c = 0; c < CF::NBN; ++c)
#pragma unroll
                for (int r = 0; r < MF::NREG; ++r) acc[a][c][r] = T(0);
        block(I0(), std::false_type(), A, B);                             // panel 2 was requested before the previous stores
        block(I1(), std::true_type(), A + 3 * stepA, B + 3 * stepB);
        const T *pa = A + 4 * stepA, *pb = B + 4 * stepB;
        for (int64_t kb = 2; kb < nkb; kb += 2) {
            if (kb + 2 == nkb) { pa = An; pb = Bn; }                      // the stream moves on to the next tile
            block(I0(), std::true_type(), pa, pb);
            pa += stepA; pb += stepB;
            block(I1(), std::true_type(), pa, pb);
            pa += stepA; pb += stepB;
        }
        gload(I0(), pa, pb);                                              // next tile's panel 2, ahead of the stores below
#pragma unroll
        for (int a = 0; a < CF::NBM; ++a)
#pragma unroll
            for (int c = 0; c < CF::NBN; ++c) {
                T *col = C + wm + a * MI + (lane % MI) + (int64_t)(wn + c * MI + MF::result_row_lane(lane)) * g.ldc;
#pragma unroll
                for (int r = 0; r < MF::NREG; ++r) {
                    T *dst = col + MF::result_row_reg(r) * g.ldc;
                    T v = alpha * acc[a][c][r];
                    if (BETA) v += beta * *dst;
                    *dst = v;
                }
            }
    };

    Loc cur = locate(b, tile);
    {   // prime the stream with the first tile's panels 0, 1 and 2
        gload(I0(), cur.A, cur.B);
        gload(I1(), cur.A + stepA, cur.B + stepB);
        PA::store(As[0], ra[0]);
        PB::store(Bs[0], rb[0]);
        __syncthreads();
        read_frags(I0(), I0(), 0);
        gload(I0(), cur.A + 2 * stepA, cur.B + 2 * stepB);
    }
    // one tile and the step to the workgroup's next one; the last tile names itself as successor
    auto step = [&]() {
        const bool more = logical + nslots < last;
        int tile2 = tile + dr;
        int64_t b2 = b + dq;
        if (tile2 >= tiles) { tile2 -= (int)tiles; ++b2; }
        const Loc nxt = more ? locate(b2, tile2) : cur;
        run_tile(cur, nxt);
        logical += nslots;
        b = b2;
        tile = tile2;
        cur = nxt;
        return more;
    };
    bool more = step();               // first tile: follows the priming above
    while (more) more = step();       // later tiles: follow a finished tile
}

// LDS panel of the direct-to-LDS kernel for an operand whose ROWS (m or n) are contiguous in memory: kept as it
// lies, [k][row], in 16-byte slots of RPS rows.  A fragment is VEC scalar reads, VEC k-rows apart, with lanes
// along the rows; the lane groups of a wave read k-rows VEC apart, which a plain layout would put on the same
// banks, so the slots of k-row k sit at position slot ^ 8 ((k / VEC) % 2): neighbouring lane groups read from
// different halves of the banks.  Only whole slots move, so the loads produce this placement by what they fetch.
template <typename MF, int ROWS, int BK>
struct RowPanel {
    typedef typename MF::T T;
    static constexpr int VEC = MF::VEC, RPS = 16 / (int)sizeof(T), SLOTS = ROWS / RPS;      // rows per slot, slots per k-row
    static constexpr int LDS_SIZE = ROWS * BK;
    static_assert(SLOTS >= 16 && RPS == VEC, "a 16-byte slot holds VEC rows; the placement flips slot bit 3");
    static __device__ __forceinline__ int flip(int k) { return ((k / VEC) & 1) << 3; }
    // what the 16-byte slot `slot16` of the panel holds: k and first row
    static __device__ __forceinline__ void source(int slot16, int &k, int &row)
    {
        k = slot16 / SLOTS;
        row = ((slot16 % SLOTS) ^ flip(k)) * RPS;
    }
    static __device__ __forceinline__ void fragment(T (&frag)[VEC], const T *lds, int row0, int kg, int lane)
    {
        constexpr int MI = MF::MI;
        const int row = row0 + (lane % MI);
        const int k = kg * MF::KGROUP + (lane / MI) * VEC;                 // (k + e) / VEC == k / VEC for e < VEC: one placement per lane
        const T *p = lds + k * ROWS + (((row / RPS) ^ flip(k)) * RPS) + row % RPS;
#pragma unroll
        for (int e = 0; e < VEC; ++e) frag[e] = p[e * ROWS];
    }
};

// Direct-to-LDS member of the streaming family: whole tiles, both operands k-contiguous, an even number of
// BK-deep panels, rows of BK elements = 128 bytes (whole cache lines).  Same walk over the tiles and the same
// fragment schedule as sbgemm_mfma_stream_kernel, but the panels travel from memory into one of two LDS stages
// without passing through registers: the panel after the next one is requested right after the barrier that
// frees its stage and has a whole panel's MFMAs to arrive.  What this saves is the staging registers and,
// measured on the register-staged kernel at 512^4, the 3 % of the run time that its LDS stores cost and part
// of the 3 % of its global loads.  The swizzled [row][k] layout (Panel<.., KC = true>) is produced by the
// choice of what each lane fetches: lane l of load j fills 16-byte slot 64 (NW j + wave) + l of the panel,
// i.e. row slot / CPR, and fetches that row's chunk (slot % CPR) ^ f(row).  An operand with m or n contiguous
// lands as [k][row] (RowPanel) and is read with lanes along the rows, one element per k.
template <typename MFT, bool A_KC, bool B_KC, bool BETA, int BK, int WM, int WN, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N, WAVES_M * WAVES_N <= 4 ? 2 : 1) void sbgemm_mfma_dma_kernel(SbArgs g, int tiles_m, int tiles_n)
{
    typedef Config<MFT, true, true, BK, WM, WN, WAVES_M, WAVES_N, 2> CF;         // k-contiguous layouts and fragment reads
    typedef typename CF::MF MF;
    typedef typename MF::T T;
    typedef typename CF::PA PA;
    typedef typename CF::PB PB;
    typedef RowPanel<MFT, CF::BM, BK> RA;
    typedef RowPanel<MFT, CF::BN, BK> RB;
    constexpr int MI = MF::MI, VEC = MF::VEC, BM = CF::BM, BN = CF::BN, KG = BK / MF::KGROUP, NW = WAVES_M * WAVES_N;
    static_assert(BK * sizeof(T) == 128 && PA::CPR == 8, "a panel row is one 128-byte line of eight chunks");
    // A row-contiguous fp32 A panel lies [k][row], so one LDS read of NBM consecutive rows at one k feeds all NBM
    // MFMA blocks of the wave if lane j of block a stands for tile row wm + NBM j + a (instead of wm + 32 a + j):
    // a quarter (half) of the read instructions, and the lane then holds NBM consecutive rows of every column,
    // which leave as one vector store.  The row <-> (block, lane) map is free as long as every k uses the same one.
    constexpr bool A_IL = !A_KC && sizeof(T) == 4 && (CF::NBM == 2 || CF::NBM == 4);
    typedef T RowVec __attribute__((ext_vector_type(CF::NBM > 1 ? CF::NBM : 2)));
    typedef T RowVecU __attribute__((ext_vector_type(CF::NBM > 1 ? CF::NBM : 2), aligned(sizeof(T))));
    static_assert((BM * 8) % (64 * NW) == 0 && (BN * 8) % (64 * NW) == 0, "whole wave loads per panel");
    constexpr int NLA = BM * 8 / (64 * NW), NLB = BN * 8 / (64 * NW);        // 16-byte loads per lane and panel
    constexpr int STAGE = PA::LDS_SIZE + PB::LDS_SIZE;                       // elements per stage: A panel, B panel
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_bytes[];
    T *lds = (T *)lds_bytes;                                                 // [stage][A | B]

    // leading dimension of a panel (row stride of a k-contiguous operand, k stride of the other kind) and the
    // element step from one panel to the next
    const int64_t ldA = A_KC ? g.rsA : g.csA, ldB = B_KC ? g.csB : g.rsB;
    const int64_t panelA = A_KC ? BK : (int64_t)BK * g.csA, panelB = B_KC ? BK : (int64_t)BK * g.rsB;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave % WAVES_M) * WM, wn = (wave / WAVES_M) * WN;
    const T alpha = (T)g.alpha, beta = (T)g.beta;
    const int64_t nkb = g.k / BK;

    const int64_t tiles = (int64_t)tiles_m * tiles_n;
    const int64_t total = tiles * g.batch0 * g.batch1;
    const int64_t nslots = (int64_t)gridDim.x / NXCD;
    const int64_t xcd = blockIdx.x % NXCD, slot = blockIdx.x / NXCD;
    const int64_t q8 = total / NXCD, r8 = total % NXCD;
    const int64_t first = xcd * q8 + (xcd < r8 ? xcd : r8);
    const int64_t last = first + q8 + (xcd < r8 ? 1 : 0);
    int64_t logical = first + slot;
    if (logical >= last) return;

    // what this lane fetches: byte offsets from the panel's first element, per load; and where its wave's loads land
    unsigned offA[NLA], offB[NLB];
#pragma unroll
    for (int j = 0; j < NLA; ++j) {
        const int slot16 = 64 * (NW * j + wave) + lane;
        int row = slot16 / 8, k = PA::swizzled(row, (slot16 % 8) * VEC);            // the swizzle is its own inverse
        if (!A_KC) RA::source(slot16, k, row);
        offA[j] = (unsigned)((A_KC ? (int64_t)row * ldA + k : (int64_t)k * ldA + row) * sizeof(T));
    }
#pragma unroll
    for (int j = 0; j < NLB; ++j) {
        const int slot16 = 64 * (NW * j + wave) + lane;
        int row = slot16 / 8, k = PB::swizzled(row, (slot16 % 8) * VEC);
        if (!B_KC) RB::source(slot16, k, row);
        offB[j] = (unsigned)((B_KC ? (int64_t)row * ldB + k : (int64_t)k * ldB + row) * sizeof(T));
    }
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)lds_bytes;
    const unsigned land = __builtin_amdgcn_readfirstlane(lds0 + wave * 1024);

    T fa[2][CF::NBM][VEC], fb[2][CF::NBN][VEC];
    typename MF::Acc acc[CF::NBM][CF::NBN];

    struct Loc { const T *A, *B; T *C; };
    auto locate = [&](int64_t b, int tile) __attribute__((always_inline)) {
        int64_t b0 = b, b1 = 0;
        if (g.batch1 != 1) { b1 = b / g.batch0; b0 = b - b1 * g.batch0; }
        const SbOff3 o1 = sb_level1(g, b1);
        const unsigned tn = (unsigned)tile / (unsigned)tiles_m, tm = (unsigned)tile - tn * (unsigned)tiles_m;
        const int64_t i0 = (int64_t)tm * BM, j0 = (int64_t)tn * BN;
        Loc l;
        l.A = (const T *)g.A + b0 * g.bsA[0] + o1.a + i0 * g.rsA;
        l.B = (const T *)g.B + b0 * g.bsB[0] + o1.b + j0 * g.csB;
        l.C = (T *)g.C + b0 * g.bsC[0] + o1.c + i0 + j0 * g.ldc;
        return l;
    };
    int64_t b = logical / tiles;
    int tile = (int)(logical - b * tiles);
    const int64_t dq = nslots / tiles;
    const int dr = (int)(nslots - dq * tiles);

    typedef std::integral_constant<int, 0> I0;
    typedef std::integral_constant<int, 1> I1;
    auto request = [&](auto st_c, const T *pa, const T *pb) __attribute__((always_inline)) {
        constexpr unsigned at = decltype(st_c)::value * STAGE * sizeof(T);
#pragma unroll
        for (int j = 0; j < NLA; ++j) dma16(land + at + j * NW * 1024, pa, offA[j]);
#pragma unroll
        for (int j = 0; j < NLB; ++j) dma16(land + at + PA::LDS_SIZE * sizeof(T) + j * NW * 1024, pb, offB[j]);
    };
    auto read_frags = [&](auto set_c, auto st_c, int kg) __attribute__((always_inline)) {
        constexpr int SET = decltype(set_c)::value, ST = decltype(st_c)::value;
        const T *As = lds + ST * STAGE, *Bs = As + PA::LDS_SIZE;
        if constexpr (A_IL) {
            const int row = wm + CF::NBM * (lane % MI);
            const int k = kg * MF::KGROUP + (lane / MI) * VEC;
            const T *p = As + k * BM + (((row / RA::RPS) ^ RA::flip(k)) * RA::RPS) + row % RA::RPS;
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const RowVec v = *(const RowVec *)(p + e * BM);
#pragma unroll
                for (int a = 0; a < CF::NBM; ++a) fa[SET][a][e] = v[a];
            }
        } else {
#pragma unroll
            for (int a = 0; a < CF::NBM; ++a) {
                if (A_KC) PA::fragment(fa[SET][a], As, wm + a * MI, kg, lane);
                else      RA::fragment(fa[SET][a], As, wm + a * MI, kg, lane);
            }
        }
#pragma unroll
        for (int c = 0; c < CF::NBN; ++c) {
            if (B_KC) PB::fragment(fb[SET][c], Bs, wn + c * MI, kg, lane);
            else      RB::fragment(fb[SET][c], Bs, wn + c * MI, kg, lane);
        }
    };
    // One panel in stage ST: KG k-groups on two alternating fragment sets.  Before the last group's MFMAs: wait
    // for the panel in flight, barrier (all waves have read this stage's last fragments), request the panel
    // after the next one into this stage, read the first fragments of the other stage.
    auto panel = [&](auto st_c, const T *pa, const T *pb) __attribute__((always_inline)) {
        constexpr int ST = decltype(st_c)::value;
        typedef std::integral_constant<int, ST> S;
        typedef std::integral_constant<int, ST ^ 1> SN;
#pragma unroll
        for (int kg = 0; kg < KG; ++kg) {
            const int fs = kg & 1;
            if (kg + 1 < KG) {
                if (fs == 0) read_frags(I1(), S(), kg + 1);
                else         read_frags(I0(), S(), kg + 1);
            } else {
                __builtin_amdgcn_sched_barrier(0);
                dma_wait<0>();
                __syncthreads();
                request(S(), pa, pb);
                __builtin_amdgcn_sched_barrier(0);
                read_frags(I0(), SN(), 0);
            }
            __builtin_amdgcn_s_setprio(2);
#pragma unroll
            for (int e = 0; e < VEC; ++e)
#pragma unroll
                for (int a = 0; a < CF::NBM; ++a)
#pragma unroll
                    for (int c = 0; c < CF::NBN; ++c) MF::mma(acc[a][c], fb[fs][c][e], fa[fs][a][e]);   // C^T = B^T A^T
            __builtin_amdgcn_s_setprio(0);
        }
    };
    // One tile: its panel 0 is complete in stage 0 with the first fragments requested, panel 1 in flight into
    // stage 1; pa / pb point at panel 2.
    auto run_tile = [&](const Loc &cur, const Loc &nxt, const T *&pa, const T *&pb) __attribute__((always_inline)) {
#pragma unroll
        for (int a = 0; a < CF::NBM; ++a)
#pragma unroll
            for (int c = 0; c < CF::NBN; ++c)
#pragma unroll
                for (int r = 0; r < MF::NREG; ++r) acc[a][c][r] = T(0);
        for (int64_t kb = 0; kb < nkb; kb += 2) {
            if (kb + 2 == nkb) { pa = nxt.A; pb = nxt.B; }                // panel kb + 2 is the next tile's first
            panel(I0(), pa, pb);
            pa += panelA; pb += panelB;
            panel(I1(), pa, pb);
            pa += panelA; pb += panelB;
        }
        T *C = cur.C;
        if constexpr (A_IL) {            // lane j: rows wm + NBM j .. + NBM - 1 of its columns, one vector per column
#pragma unroll
            for (int c = 0; c < CF::NBN; ++c) {
                T *col = C + wm + CF::NBM * (lane % MI) + (int64_t)(wn + c * MI + MF::result_row_lane(lane)) * g.ldc;
#pragma unroll
                for (int r = 0; r < MF::NREG; ++r) {
                    T *dst = col + MF::result_row_reg(r) * g.ldc;
                    RowVec v;
#pragma unroll
                    for (int a = 0; a < CF::NBM; ++a) v[a] = alpha * acc[a][c][r];
                    if (BETA) {
                        const RowVec old = *(const RowVecU *)dst;
#pragma unroll
                        for (int a = 0; a < CF::NBM; ++a) v[a] += beta * old[a];
                    }
                    *(RowVecU *)dst = v;
                }
            }
            return;
        }
#pragma unroll
        for (int a = 0; a < CF::NBM; ++a)
#pragma unroll
            for (int c = 0; c < CF::NBN; ++c) {
                T *col = C + wm + a * MI + (lane % MI) + (int64_t)(wn + c * MI + MF::result_row_lane(lane)) * g.ldc;
#pragma unroll
                for (int r = 0; r < MF::NREG; ++r) {
                    T *dst = col + MF::result_row_reg(r) * g.ldc;
                    T v = alpha * acc[a][c][r];
                    if (BETA) v += beta * *dst;
                    *dst = v;
                }
            }
    };

    Loc cur = locate(b, tile);
    const T *pa = cur.A + 2 * panelA, *pb = cur.B + 2 * panelB;
    request(I0(), cur.A, cur.B);
    request(I1(), cur.A + panelA, cur.B + panelB);
    dma_wait<NLA + NLB>();                 // panel 0 has landed; panel 1 may still be under way
    __syncthreads();
    read_frags(I0(), I0(), 0);
    bool more = true;
    while (more) {
        more = logical + nslots < last;
        int tile2 = tile + dr;
        int64_t b2 = b + dq;
        if (tile2 >= tiles) { tile2 -= (int)tiles; ++b2; }
        const Loc nxt = more ? locate(b2, tile2) : cur;       // the last tile names itself as successor: panels that are never used
        run_tile(cur, nxt, pa, pb);
        logical += nslots;
        b = b2;
        tile = tile2;
        cur = nxt;
    }
    dma_wait<0>();                         // nothing of this workgroup may still be writing LDS when it ends
}

// Launch `kernel` with as many workgroups as can be resident at once (a multiple of the XCD
// count), or fewer if there are fewer tiles.  The residency of a kernel is asked once per device.
template <typename K, typename... Extra>
hipError_t launch_persistent(K kernel, int nthreads, int64_t total_tiles, hipStream_t stream, const SbArgs &a, int tm, int tn, Extra... extra)
{
    int resident = 0;
    const hipError_t e = sb_resident_workgroups((const void *)kernel, nthreads, &resident);
    if (e != hipSuccess) return e;
    int64_t grid = total_tiles < resident ? total_tiles : resident;
    grid = (grid + NXCD - 1) / NXCD * NXCD;
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(nthreads), 0, stream, a, tm, tn, extra...);
    return hipGetLastError();
}

// The direct-to-LDS kernel of a configuration: whole tiles, each operand k-contiguous or row-contiguous, an even
// number of BK-deep panels, offsets inside a panel that fit the 32-bit lane offsets of its loads.
template <typename MFT, int BK, int WM, int WN, int WAVES_M, int WAVES_N>
bool dma_applies(const SbArgs &a)
{
    const int64_t most = (int64_t)1 << 21;
    const bool a_ok = a.csA == 1 || a.rsA == 1, b_ok = a.rsB == 1 || a.csB == 1;
    return a_ok && b_ok && a.m % (WM * WAVES_M) == 0 && a.n % (WN * WAVES_N) == 0 && a.k % (2 * BK) == 0 &&
           a.rsA <= most && a.csA <= most && a.rsB <= most && a.csB <= most;
}

// (one function per kernel: the set-up flags below belong to that kernel alone)
template <typename MFT, bool A_KC, bool B_KC, bool BETA, int BK, int WM, int WN, int WAVES_M, int WAVES_N>
hipError_t launch_dma_kernel(const SbArgs &a, hipStream_t stream)
{
    typedef typename MFT::T T;
    constexpr int BM = WM * WAVES_M, BN = WN * WAVES_N, NT = 64 * WAVES_M * WAVES_N;
    const int lds_bytes = 2 * (BM + BN) * BK * (int)sizeof(T);
    const int64_t tiles_m = a.m / BM, tiles_n = a.n / BN;
    const int64_t total = tiles_m * tiles_n * a.batch0 * a.batch1;
    if (total <= 0) return hipSuccess;
    if (total >= (int64_t)1 << 31) return hipErrorInvalidConfiguration;
    auto kernel = sbgemm_mfma_dma_kernel<MFT, A_KC, B_KC, BETA, BK, WM, WN, WAVES_M, WAVES_N>;
    static std::atomic<int> resident_of[SB_MAX_DEVICES] = {};          // 0: this device has not been set up for the kernel yet
    const int dev = sb_current_device();
    int resident = resident_of[dev];
    if (resident == 0) {
        int per_cu = 0, cus = 0;
        hipError_t e = hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, NT, lds_bytes);
        if (e != hipSuccess) return e;
        if (per_cu < 1 || cus < 1) return hipErrorInvalidConfiguration;
        resident = per_cu * cus;
        resident_of[dev] = resident;
    }
    int64_t grid = total < resident ? total : resident;
    grid = (grid + NXCD - 1) / NXCD * NXCD;
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(NT), lds_bytes, stream, a, (int)tiles_m, (int)tiles_n);
    return hipGetLastError();
}

template <typename MFT, int BK, int WM, int WN, int WAVES_M, int WAVES_N>
hipError_t launch_dma(const SbArgs &a, hipStream_t stream)
{
    const bool ak = a.csA == 1, bk = a.rsB == 1, b0 = a.beta == 0.0;
#define SB_DMA(AK, BKC) (b0 ? launch_dma_kernel<MFT, AK, BKC, false, BK, WM, WN, WAVES_M, WAVES_N>(a, stream) \
                            : launch_dma_kernel<MFT, AK, BKC, true, BK, WM, WN, WAVES_M, WAVES_N>(a, stream))
    if (ak && bk)  return SB_DMA(true, true);
    if (ak && !bk) return SB_DMA(true, false);
    if (!ak && bk) return SB_DMA(false, true);
    return SB_DMA(false, false);
#undef SB_DMA
}

// STREAM_ONLY: the caller has checked that the problem is made of whole tiles (stream_applies), so
// only the streaming kernels of this configuration are instantiated.
template <typename MFT, int BK, int WM, int WN, int WAVES_M, int WAVES_N, int GD = 2, bool STREAM_ONLY = false>
hipError_t launch(const SbArgs &a, hipStream_t stream)
{
    typedef MFT T;
    constexpr int BM = WM * WAVES_M, BN = WN * WAVES_N, NT = 64 * WAVES_M * WAVES_N;
    const int64_t tiles_m = (a.m + BM - 1) / BM, tiles_n = (a.n + BN - 1) / BN;
    const int64_t total = tiles_m * tiles_n * a.batch0 * a.batch1;
    if (total <= 0) return hipSuccess;
    if (total >= (int64_t)1 << 31) return hipErrorInvalidConfiguration;
    const bool a_kc = (a.csA == 1), b_kc = (a.rsB == 1);
    // per operand (bit 0: A, bit 1: B): its panels may be read as 16-byte vectors.  The hardware
    // reads such a vector at any element-aligned address, so leading dimensions and offsets need
    // not be multiples of the vector length.
    const int vec_ok = 3;
    const int tm = (int)tiles_m, tn = (int)tiles_n;
    // whole tiles, aligned operands, an even number (>= 4) of k blocks: the streaming kernel
    if (vec_ok == 3 && a.m % BM == 0 && a.n % BN == 0 && a.k % (2 * BK) == 0 && a.k >= 4 * BK) {
#define STREAM(AK, BKC)                                                                                                                  \
    (a.beta == 0.0 ? launch_persistent(sbgemm_mfma_stream_kernel<T, AK, BKC, false, BK, WM, WN, WAVES_M, WAVES_N>, NT, total, stream, a, tm, tn) \
                   : launch_persistent(sbgemm_mfma_stream_kernel<T, AK, BKC, true, BK, WM, WN, WAVES_M, WAVES_N>, NT, total, stream, a, tm, tn))
        if (a_kc && b_kc)        return STREAM(true, true);
        else if (a_kc && !b_kc)  return STREAM(true, false);
        else if (!a_kc && b_kc)  return STREAM(false, true);
        return STREAM(false, false);
#undef STREAM
    }
    if constexpr (STREAM_ONLY) return hipErrorInvalidValue;
    else {
    if (a_kc && b_kc)        return launch_persistent(sbgemm_mfma_kernel<T, true, true, BK, WM, WN, WAVES_M, WAVES_N, GD>, NT, total, stream, a, tm, tn, vec_ok);
    else if (a_kc && !b_kc)  return launch_persistent(sbgemm_mfma_kernel<T, true, false, BK, WM, WN, WAVES_M, WAVES_N, GD>, NT, total, stream, a, tm, tn, vec_ok);
    else if (!a_kc && b_kc)  return launch_persistent(sbgemm_mfma_kernel<T, false, true, BK, WM, WN, WAVES_M, WAVES_N, GD>, NT, total, stream, a, tm, tn, vec_ok);
    return launch_persistent(sbgemm_mfma_kernel<T, false, false, BK, WM, WN, WAVES_M, WAVES_N, GD>, NT, total, stream, a, tm, tn, vec_ok);
    }
}

// Whole BM x BN tiles and an even number (>= 4) of BK-deep k blocks: what the
// streaming kernels need (the same test as inside launch()).
template <typename MFT>
bool stream_applies(const SbArgs &a, int BM, int BN, int BK)
{
    return a.m % BM == 0 && a.n % BN == 0 && a.k % (2 * BK) == 0 && a.k >= 4 * BK;
}

}  // namespace

// Estimated run time of a problem cut into `tiles` equal tiles, in units of one 128 x 128 tile on a
// compute unit of its own: the busiest of the 256 compute units gets ceil(tiles / 256) tiles (two
// workgroups that share a unit take turns on its matrix core, so they count like one after the
// other), each `area` times a 128 x 128 tile and `gain` times faster per flop.
double sb_tile_time(int64_t tiles, double area, double gain)
{
    const int64_t units = 256;
    return (double)((tiles + units - 1) / units) * area / gain;
}

// N and T operands only: one of the two strides of each operand must be 1.
bool sb_mfma_supports(sb_dtype dt, const SbArgs &a)
{
    if (sb_mfma_exa_supports(dt, a)) return true;           // extended operation on the first operand
    if (a.k <= 0) return false;
    const bool a_ok = (a.csA == 1) || (a.rsA == 1);
    const bool b_ok = (a.rsB == 1) || (a.csB == 1);
    if (!a_ok || !b_ok) return false;
    // a k-contiguous operand with a single row or a single k is also "row contiguous": either view works
    const int64_t tiles = ((a.m + 63) / 64) * ((a.n + 63) / 64);       // smallest tile used below
    // fp32 / fp64 run persistent workgroups (32-bit tile counters); the plain bf16 kernel takes one
    // workgroup per tile in a one-dimensional grid
    const int64_t most = dt == SB_BF16 ? sb_max_grid_x(256) : ((int64_t)1 << 31) - 1;
    return tiles * a.batch0 * a.batch1 <= most;
}

bool sb_mfma_preferred(sb_dtype dt, const SbArgs &a)
{
    if (sb_mfma_exa_supports(dt, a)) return a.m >= 16 && a.n >= 16 && a.k >= 8;
    // Nearly every N/T problem the thin and tiny kernels leave.
    // m, n >= 32, any k: with a short k the call is bound by writing C, and the MFMA kernel's stores
    // of whole 128-byte runs beat the general kernel by 1.6x even at k = 1 (rank-1 updates).
    if (a.m >= 32 && a.n >= 32) return true;
    // a factor matrix against a tensor unfolding: the long tiles stream the big operand
    const int64_t hi = a.m < a.n ? a.n : a.m;
    if (hi >= 256) return true;
    // Smaller shapes, where most of a 64 x 64 tile is padding (m = 10, n = 100): the vector loads
    // and the matrix core are still 1.1-2.2x (bf16: 1.3-3.5x) ahead of the general kernel's scalar
    // loads and vector-ALU products unless k is short (k < 32: the general kernel is 1.2-1.5x ahead).
    return dt == SB_BF16 || a.k >= 32;
}

hipError_t sb_launch_mfma(sb_dtype dt, const SbArgs &a, hipStream_t stream)
{
    if (sb_mfma_exa_supports(dt, a)) return sb_launch_mfma_exa(dt, a, stream);
    // a problem of few 128 x 128 tiles leaves most compute units idle: 64 x 64 tiles spread it over
    // four times as many workgroups
    const int64_t tiles128 = ((a.m + 127) / 128) * ((a.n + 127) / 128) * a.batch0 * a.batch1;
    const bool few_tiles = tiles128 < 128;
    // and so do extents just above a multiple of 128 (300 x 300: 128 x 128 tiles compute 1.64 times
    // the result's area, 64 x 64 tiles 1.14 times)
    auto padded = [](int64_t x, int64_t t) { return (x + t - 1) / t * t; };
    const bool much_padding = (double)(padded(a.m, 128) * padded(a.n, 128)) > 1.15 * (double)(padded(a.m, 64) * padded(a.n, 64));
    const bool small_tiles = a.m <= 64 || a.n <= 64 || few_tiles || much_padding;
    switch (dt) {
    case SB_F32:
        // a factor matrix against a tensor unfolding: bound by streaming the big operand, so the
        // tile is long in that operand's direction (big panels in flight) and one MFMA block wide
        if (a.n <= 32 && a.m >= 256) return launch<MfmaF32x32, 32, 32, 32, 4, 1>(a, stream);     // 128 x 32 tiles, 4 waves
        if (a.m <= 32 && a.n >= 256) return launch<MfmaF32x32, 32, 32, 32, 1, 4>(a, stream);     // 32 x 128 tiles
        if (small_tiles) {                                                               // 64 x 64 tiles
            if (dma_applies<MfmaF32x32, 32, 32, 32, 2, 2>(a) && a.k >= 128) return launch_dma<MfmaF32x32, 32, 32, 32, 2, 2>(a, stream);
            return launch<MfmaF32x32, 16, 32, 32, 2, 2>(a, stream);
        }
        // whole 256 x 256 or 128 x 256 tiles: eight waves of 128 x 64 or 64 x 64 (fewer panel loads per
        // flop and fewer, longer tiles: 4-5 % and 2-3 % over the 128 x 128 tiles at 512^4), unless the
        // bigger tiles would leave compute units idle (few tiles, or a last round that is mostly empty)
        {
            const int64_t batch = a.batch0 * a.batch1;
            const double t128 = sb_tile_time(tiles128, 1.0, 1.0);
            // (256 x 256 only for a long k and more than one round of tiles: a compute unit that gets a single tile runs its
            // loads, products and stores one after the other, and short tiles end too often; there 128 x 256 tiles, two
            // workgroups' worth per compute unit, are 2-9 % faster: 256^3 x 256 74.6 -> 70.5 us)
            const int64_t tiles256 = (a.m / 256) * (a.n / 256) * batch;
            if (stream_applies<MfmaF32x32>(a, 256, 256, 16) && tiles256 > 256 && a.k >= 256 && sb_tile_time(tiles256, 4.0, 1.04) <= t128) {
#ifndef SB_F32_NO_DMA
                if (dma_applies<MfmaF32x32, 32, 128, 64, 2, 4>(a)) return launch_dma<MfmaF32x32, 32, 128, 64, 2, 4>(a, stream);
#endif
                return launch<MfmaF32x32, 16, 128, 64, 2, 4, 2, true>(a, stream);
            }
            if (stream_applies<MfmaF32x32>(a, 128, 256, 16) && sb_tile_time((a.m / 128) * (a.n / 256) * batch, 2.0, 1.02) <= t128) {
                if (dma_applies<MfmaF32x32, 32, 64, 64, 2, 4>(a)) return launch_dma<MfmaF32x32, 32, 64, 64, 2, 4>(a, stream);
                return launch<MfmaF32x32, 16, 64, 64, 2, 4, 2, true>(a, stream);
            }
        }
        if (dma_applies<MfmaF32x32, 32, 64, 64, 2, 2>(a)) return launch_dma<MfmaF32x32, 32, 64, 64, 2, 2>(a, stream);
        return launch<MfmaF32x32, 16, 64, 64, 2, 2>(a, stream);                                  // 128 x 128 tiles
    case SB_F64:
        if (a.n <= 32 && a.m >= 256) return launch<MfmaF64x16, 16, 32, 32, 4, 1>(a, stream);     // 128 x 32 tiles, 4 waves
        if (a.m <= 32 && a.n >= 256) return launch<MfmaF64x16, 16, 32, 32, 1, 4>(a, stream);     // 32 x 128 tiles
        if (small_tiles) return launch<MfmaF64x16, 16, 32, 32, 2, 2>(a, stream);      // (direct-to-LDS loads: no gain on 64 x 64 fp64 tiles)
#ifndef SB_F64_NO_DMA
        if (dma_applies<MfmaF64x16, 16, 32, 32, 4, 4>(a)) return launch_dma<MfmaF64x16, 16, 32, 32, 4, 4>(a, stream);
#endif
        return launch<MfmaF64x16, 16, 32, 32, 4, 4>(a, stream);                                 // 128 x 128 tiles, 16 waves
    case SB_BF16: return sb_launch_mfma_bf16(a, stream);
    default: break;
    }
    return hipErrorInvalidValue;
}
