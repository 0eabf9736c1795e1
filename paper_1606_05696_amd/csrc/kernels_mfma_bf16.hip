// MFMA-tiled StridedBatchedGemm for bf16 inputs with fp32 accumulation and bf16 output.
//
// Same organisation as the fp32/fp64 kernel (one workgroup of four waves per C tile, batch folded
// into the grid, double-buffered LDS panels, XCD-aware tile order, C^T trick for coalesced
// stores), built on v_mfma_f32_32x32x16_bf16.  That instruction wants 8 consecutive k per lane
// for both operands (lane l holds X[l%32][8*(l/32) .. +7]):
//   k contiguous operand (A with T, B with N): LDS [row][k], one 16-byte LDS read per fragment;
//   m/n contiguous operand (A with N, B with T): LDS [k][row]; the 8 k of a fragment are gathered
//     with 2-byte LDS reads (conflict-free: the lanes of a read run along the row dimension).
// The epilogue rounds alpha*acc + beta*C to bf16 (nearest even).
// Three members: the plain kernel above (any size and alignment), the streaming kernel (whole 128 x 128 or
// 256 x 256 tiles, persistent workgroups, panels staged through registers; an m/n-contiguous operand is
// transposed in registers into the k-contiguous LDS layout), and the direct-to-LDS kernel (256 x 256 tiles,
// both operands k-contiguous).
#include "sb_device.h"
#include "sb_internal.h"

#include <atomic>

#include <type_traits>

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short u16x8u __attribute__((ext_vector_type(8), aligned(2)));      // global loads: any element address

constexpr int NTHREADS = 256;
constexpr int NXCD = 8;
constexpr int BK = 32;          // two MFMA k-steps of 16 per panel

// SWZ (k-contiguous panels only): rows are stored unpadded and the 16-byte chunk c of row r sits at
// chunk c ^ f(r), f(r) = (r / rows-per-256-bytes) mod chunks-per-row.  Sixteen lanes that write
// consecutive chunks then cover 256 contiguous bytes, and sixteen lanes that read the same chunk
// of consecutive rows (an MFMA fragment) hit sixteen different bank groups: neither conflicts.
// (With padding the reads are conflict-free but a store wraps onto the banks of the row 3 above.)
template <bool KC, int ROWS, int BK = 32, bool SWZ = false, int NT = NTHREADS>
struct PanelBf16 {
    static_assert(!SWZ || KC, "the swizzle is for k-contiguous panels");
    static constexpr int NVEC = ROWS * BK / 8 / NT;             // 16-byte vectors per lane
    static constexpr int LDS_LD = SWZ ? BK : (KC ? BK : ROWS) + 8;    // padded by 16 bytes unless swizzled
    static constexpr int CPR = BK / 8;                                // 16-byte chunks per row
    static __device__ __forceinline__ int swizzled(int row, int k)   // k a multiple of 8
    {
        return SWZ ? (((k >> 3) ^ ((row / (16 / CPR)) & (CPR - 1))) << 3) : k;
    }
    static constexpr int LDS_SIZE = (KC ? ROWS : BK) * LDS_LD;
    static_assert(ROWS * BK % (8 * NT) == 0, "panel must split evenly over the lanes");

    static __device__ __forceinline__ void coords(int f, int &row, int &k)
    {
        if (KC) { row = f / (BK / 8); k = (f % (BK / 8)) * 8; }
        else    { k = f / (ROWS / 8); row = (f % (ROWS / 8)) * 8; }
    }

    static __device__ __forceinline__ void load(u16x8 (&v)[NVEC], const uint16_t *p, int64_t ld, int64_t rows_left, int64_t k_left, bool vec_ok)
    {
#pragma unroll
        for (int q = 0; q < NVEC; ++q) {
            int row, k;
            coords((int)threadIdx.x + NT * q, row, k);
            const uint16_t *src = KC ? p + (int64_t)row * ld + k : p + (int64_t)k * ld + row;
            const bool inside = KC ? (row < rows_left && k + 8 <= k_left) : (row + 8 <= rows_left && k < k_left);
            if (vec_ok && inside) {
                v[q] = *(const u16x8u *)src;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const bool ok = KC ? (row < rows_left && k + e < k_left) : (row + e < rows_left && k < k_left);
                    v[q][e] = ok ? src[e] : (uint16_t)0;
                }
            }
        }
    }

    // whole panel inside the matrix, every vector aligned: no branch, the loads stay countable
    static __device__ __forceinline__ void load_plain(u16x8 (&v)[NVEC], const uint16_t *p, int64_t ld)
    {
#pragma unroll
        for (int q = 0; q < NVEC; ++q) {
            int row, k;
            coords((int)threadIdx.x + NT * q, row, k);
            v[q] = *(const u16x8u *)(KC ? p + (int64_t)row * ld + k : p + (int64_t)k * ld + row);
        }
    }

    static __device__ __forceinline__ void store(uint16_t *lds, const u16x8 (&v)[NVEC])
    {
#pragma unroll
        for (int q = 0; q < NVEC; ++q) {
            int row, k;
            coords((int)threadIdx.x + NT * q, row, k);
            uint16_t *dst = KC ? lds + row * LDS_LD + swizzled(row, k) : lds + k * LDS_LD + row;
            *(u16x8 *)dst = v[q];
        }
    }

    // operand fragment of the 32-row block starting at row0 for MFMA k-step ks (16 k)
    static __device__ __forceinline__ bf16x8 fragment(const uint16_t *lds, int row0, int ks, int lane)
    {
        const int row = row0 + (lane & 31);
        const int k = ks * 16 + (lane >> 5) * 8;
        u16x8 v;
        if (KC) {
            v = *(const u16x8 *)(lds + row * LDS_LD + swizzled(row, k));
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = lds[(k + e) * LDS_LD + row];
        }
        return __builtin_bit_cast(bf16x8, v);
    }
};

// The same swizzled [row][k] panel for an operand whose ROWS (m or n) are contiguous in memory: it is
// transposed on the way in.  A lane loads NVEC vectors of 8 rows at NVEC consecutive k, transposes the
// 8 x NVEC block in registers and writes, for each of its 8 rows, the NVEC k as one 4- or 8-byte piece of
// that row's 16-byte chunk; fragments are read exactly as from a k-contiguous panel.
// Lane -> block: the k index runs fastest (BK / NVEC = 16 lanes share 8 rows), because that is what the
// LDS writes need: the 16 lanes' pieces are one whole row, i.e. consecutive banks, whereas lanes on the
// same k and rows 8 apart would all hit the same bank.  Where a row is shorter than the 32 banks (BK = 32:
// 64 bytes), neighbouring groups of 8 rows write their even and odd rows in opposite order, so that two
// groups together cover all banks.  The price is global loads in runs of 64 bytes instead of 512.
template <int ROWS, int BK, int NT>
struct PanelBf16T {
    typedef PanelBf16<true, ROWS, BK, true, NT> Kc;           // layout and fragment reads
    static constexpr int NVEC = Kc::NVEC;
    static constexpr int LDS_SIZE = Kc::LDS_SIZE;
    static constexpr int KQ = BK / NVEC;                       // blocks along k
    static constexpr bool FLIP = BK * 2 < 128;
    static_assert(NVEC == 2 || NVEC == 4, "a lane's block is 8 rows x 2 or 4 k");
    static_assert((ROWS / 8) * KQ == NT, "one block per lane");

    static __device__ __forceinline__ void load_plain(u16x8 (&v)[NVEC], const uint16_t *p, int64_t ld)
    {
        const int f = (int)threadIdx.x, kq = f % KQ, rg = f / KQ;
#pragma unroll
        for (int q = 0; q < NVEC; ++q) v[q] = *(const u16x8u *)(p + (int64_t)(kq * NVEC + q) * ld + rg * 8);
    }

    static __device__ __forceinline__ void store(uint16_t *lds, const u16x8 (&v)[NVEC])
    {
        typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
        typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
        const int f = (int)threadIdx.x, kq = f % KQ, rg = f / KQ;
        const int k0 = kq * NVEC;                              // first k of this lane's block
        const bool odd = FLIP && (rg & 1);
        u32x4 d[NVEC];                                         // dword t of d[q]: rows 2t (low half) and 2t+1 at k0 + q
#pragma unroll
        for (int q = 0; q < NVEC; ++q) d[q] = __builtin_bit_cast(u32x4, v[q]);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            u32x2 even, oddp;                                  // the pieces of rows 2t and 2t+1 (NVEC == 2: first word only)
            even[0] = (d[0][t] & 0xffffu) | (d[1][t] << 16);
            oddp[0] = (d[0][t] >> 16) | (d[1][t] & 0xffff0000u);
            if (NVEC == 4) {
                even[1] = (d[2][t] & 0xffffu) | (d[3][t] << 16);
                oddp[1] = (d[2][t] >> 16) | (d[3][t] & 0xffff0000u);
            }
#pragma unroll
            for (int h = 0; h < 2; ++h) {                      // first the even row (the odd one in flipped groups)
                const int row = rg * 8 + 2 * t + (odd ? 1 - h : h);
                const u32x2 piece = (h == 0) == !odd ? even : oddp;
                uint16_t *dst = lds + row * Kc::LDS_LD + Kc::swizzled(row, k0 & ~7) + (k0 & 7);
                if (NVEC == 2) *(uint32_t *)dst = piece[0];
                else           *(u32x2 *)dst = piece;
            }
        }
    }

    static __device__ __forceinline__ bf16x8 fragment(const uint16_t *lds, int row0, int ks, int lane)
    {
        return Kc::fragment(lds, row0, ks, lane);
    }
};

// WT: wave tile edge (64 -> 128x128 workgroup tile, 32 -> 64x64)
template <bool A_KC, bool B_KC, int WT>
__global__ __launch_bounds__(NTHREADS) void sbgemm_mfma_bf16_kernel(SbArgs g, int tiles_m, int tiles_n, int vec_ok)
{
    constexpr int BM = 2 * WT, BN = 2 * WT, NB = WT / 32;
    typedef PanelBf16<A_KC, BM> PA;
    typedef PanelBf16<B_KC, BN> PB;
    __shared__ __attribute__((aligned(16))) uint16_t As[2][PA::LDS_SIZE];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][PB::LDS_SIZE];

    // hardware deals consecutive workgroup ids to the 8 XCDs in turn: renumber so that each XCD
    // owns a contiguous range of tiles and batches
    const int64_t total = (int64_t)gridDim.x;
    const int64_t bid = blockIdx.x;
    const int64_t q8 = total / NXCD, r8 = total % NXCD;
    const int64_t xcd = bid % NXCD, slot = bid / NXCD;
    const int64_t logical = xcd * q8 + (xcd < r8 ? xcd : r8) + slot;
    const int64_t tiles = (int64_t)tiles_m * tiles_n;
    const int64_t b = logical / tiles;
    const int tile = (int)(logical - b * tiles);
    const int64_t b1 = b / g.batch0, b0 = b - b1 * g.batch0;
    const SbOff3 o1 = sb_level1(g, b1);
    const int tm = tile % tiles_m, tn = tile / tiles_m;
    const int64_t i0 = (int64_t)tm * BM, j0 = (int64_t)tn * BN;

    const uint16_t *A = (const uint16_t *)g.A + b0 * g.bsA[0] + o1.a + i0 * g.rsA;
    const uint16_t *B = (const uint16_t *)g.B + b0 * g.bsB[0] + o1.b + j0 * g.csB;
    uint16_t *C = (uint16_t *)g.C + b0 * g.bsC[0] + o1.c;
    const int64_t ldA = A_KC ? g.rsA : g.csA;
    const int64_t ldB = B_KC ? g.csB : g.rsB;
    const int64_t kstepA = A_KC ? 1 : g.csA;
    const int64_t kstepB = B_KC ? 1 : g.rsB;
    const int64_t m_left = g.m - i0, n_left = g.n - j0;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave & 1) * WT, wn = (wave >> 1) * WT;

    f32x16 acc[NB][NB];
#pragma unroll
    for (int a = 0; a < NB; ++a)
#pragma unroll
        for (int c = 0; c < NB; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][c][r] = 0.f;

    u16x8 ra[PA::NVEC], rb[PB::NVEC];
    const int64_t nkb = (g.k + BK - 1) / BK;
    if (nkb > 0) {
        PA::load(ra, A, ldA, m_left, g.k, vec_ok & 1);
        PB::load(rb, B, ldB, n_left, g.k, vec_ok & 2);
        PA::store(As[0], ra);
        PB::store(Bs[0], rb);
    }
    __syncthreads();
    for (int64_t kb = 0; kb < nkb; ++kb) {
        const int cur = (int)(kb & 1);
        const bool more = kb + 1 < nkb;
        if (more) {
            const int64_t k0 = (kb + 1) * BK;
            PA::load(ra, A + k0 * kstepA, ldA, m_left, g.k - k0, vec_ok & 1);
            PB::load(rb, B + k0 * kstepB, ldB, n_left, g.k - k0, vec_ok & 2);
        }
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fa[NB], fb[NB];
#pragma unroll
            for (int a = 0; a < NB; ++a) fa[a] = PA::fragment(As[cur], wm + a * 32, ks, lane);
#pragma unroll
            for (int c = 0; c < NB; ++c) fb[c] = PB::fragment(Bs[cur], wn + c * 32, ks, lane);
#pragma unroll
            for (int a = 0; a < NB; ++a)
#pragma unroll
                for (int c = 0; c < NB; ++c)      // C^T = B^T A^T: lanes run along rows of C
                    acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[c], fa[a], acc[a][c], 0, 0, 0);
        }
        if (more) {
            PA::store(As[cur ^ 1], ra);
            PB::store(Bs[cur ^ 1], rb);
        }
        __syncthreads();
    }

    const float alpha = (float)g.alpha, beta = (float)g.beta;
#pragma unroll
    for (int a = 0; a < NB; ++a) {
        const int64_t i = i0 + wm + a * 32 + (lane & 31);
        if (i >= g.m) continue;
#pragma unroll
        for (int c = 0; c < NB; ++c) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t j = j0 + wn + c * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (j >= g.n) continue;
                uint16_t *dst = C + i + j * g.ldc;
                float v = alpha * acc[a][c][r];
                if (beta != 0.f) v += beta * sb_bf16_to_f32(*dst);
                *dst = sb_f32_to_bf16(v);
            }
        }
    }
}

// Streaming variant for problems made of whole 128 x 128 tiles with both operands k-contiguous
// (A with T, B with N), aligned, k a multiple of 128: persistent workgroups walk over their tiles
// and the panel stream (64 k per panel, two panels in flight in registers, LDS double buffer) never
// drains at a tile boundary.  The schedule is the one of the fp32 / fp64 streaming kernel:
//   - while the last panels of a tile are multiplied, the first panels of the workgroup's next tile
//     are already requested, and the loads of its third panel are issued BEFORE the finished tile's
//     stores (loads and stores share one in-order counter);
//   - the LDS store of the next panel sits between the MFMAs of the second-to-last k-group, the
//     barrier and the first fragment read of the new panel before the last k-group's MFMAs;
//   - the tile body exists twice (first tile after the priming, later tiles in a loop) and
//     beta != 0 is a kernel of its own, so that no two paths with different numbers of outstanding
//     memory operations meet.
// Every lambda is forced inline: a closure that is called holds the register arrays by address,
// which would put them in scratch memory.
// NBM x NBN: MFMA blocks per wave tile, WAVES_M x WAVES_N waves.  2 x 2 blocks on 2 x 2 waves (128 x 128
// workgroup tile, two workgroups per compute unit) read one LDS fragment per MFMA, which makes LDS
// bandwidth the limit at about two thirds of the matrix peak; 4 x 2 blocks on 2 x 4 waves (256 x 256
// tile, one workgroup of 512 lanes per compute unit, still two waves per SIMD) read three quarters
// of a fragment per MFMA and half the panel bytes per flop.  (4 x 4 blocks on 2 x 2 waves, with 256
// accumulator registers and one wave per SIMD, were slower: nothing hides a wave's own stalls.)
// SBK: k per panel (64 for 2 x 2 blocks; 32 for 4 x 2, whose staging registers must share 256 with 128 accumulators).
template <bool BETA, int NBM, int NBN, int SBK, int WAVES_M = 2, int WAVES_N = 2, bool A_KC = true, bool B_KC = true>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N, (NBM * NBN <= 4 && WAVES_M * WAVES_N == 4) ? 2 : 1)
void sbgemm_bf16_stream_kernel(SbArgs g, int tiles_m, int tiles_n)
{
    constexpr int WM = 32 * NBM, WN = 32 * NBN, TM = WAVES_M * WM, TN = WAVES_N * WN, NT = 64 * WAVES_M * WAVES_N;
    typedef typename std::conditional<A_KC, PanelBf16<true, TM, SBK, true, NT>, PanelBf16T<TM, SBK, NT>>::type PA;
    typedef typename std::conditional<B_KC, PanelBf16<true, TN, SBK, true, NT>, PanelBf16T<TN, SBK, NT>>::type PB;
    constexpr int KG = SBK / 16;                 // MFMA k-steps per panel (even: two fragment sets alternate)
    __shared__ __attribute__((aligned(16))) uint16_t As[2][PA::LDS_SIZE];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][PB::LDS_SIZE];

    // leading dimension of a panel (row stride of a k-contiguous operand, k stride of the other kind) and the
    // element step from one k to the next
    const int64_t ldA = A_KC ? g.rsA : g.csA, ldB = B_KC ? g.csB : g.rsB;
    const int64_t panelA = A_KC ? SBK : (int64_t)SBK * g.csA, panelB = B_KC ? SBK : (int64_t)SBK * g.rsB;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave % WAVES_M) * WM, wn = (wave / WAVES_M) * WN;
    const float alpha = (float)g.alpha, beta = (float)g.beta;
    const int64_t nkb = g.k / SBK;

    const int64_t tiles = (int64_t)tiles_m * tiles_n;
    const int64_t total = tiles * g.batch0 * g.batch1;
    const int64_t nslots = (int64_t)gridDim.x / NXCD;           // the launcher makes gridDim.x a multiple of 8
    const int64_t xcd = blockIdx.x % NXCD, slot = blockIdx.x / NXCD;
    const int64_t q8 = total / NXCD, r8 = total % NXCD;
    const int64_t first = xcd * q8 + (xcd < r8 ? xcd : r8);
    const int64_t last = first + q8 + (xcd < r8 ? 1 : 0);
    int64_t logical = first + slot;
    if (logical >= last) return;

    u16x8 ra[2][PA::NVEC], rb[2][PB::NVEC];
    bf16x8 fa[2][NBM], fb[2][NBN];
    f32x16 acc[NBM][NBN];

    struct Loc { const uint16_t *A, *B; uint16_t *C; };
    auto locate = [&](int64_t b, int tile) __attribute__((always_inline)) {
        int64_t b0 = b, b1 = 0;
        if (g.batch1 != 1) { b1 = b / g.batch0; b0 = b - b1 * g.batch0; }
        const SbOff3 o1 = sb_level1(g, b1);
        const unsigned tn = (unsigned)tile / (unsigned)tiles_m, tm = (unsigned)tile - tn * (unsigned)tiles_m;
        const int64_t i0 = (int64_t)tm * TM, j0 = (int64_t)tn * TN;
        Loc l;
        l.A = (const uint16_t *)g.A + b0 * g.bsA[0] + o1.a + i0 * g.rsA;
        l.B = (const uint16_t *)g.B + b0 * g.bsB[0] + o1.b + j0 * g.csB;
        l.C = (uint16_t *)g.C + b0 * g.bsC[0] + o1.c + i0 + j0 * g.ldc;
        return l;
    };
    int64_t b = logical / tiles;
    int tile = (int)(logical - b * tiles);
    const int64_t dq = nslots / tiles;
    const int dr = (int)(nslots - dq * tiles);

    auto gload = [&](auto set, const uint16_t *pa, const uint16_t *pb) __attribute__((always_inline)) {
        PA::load_plain(ra[set], pa, ldA);
        PB::load_plain(rb[set], pb, ldB);
    };
    auto read_frags = [&](auto set, auto buf, int kg) __attribute__((always_inline)) {
#pragma unroll
        for (int a = 0; a < NBM; ++a) fa[set][a] = PA::fragment(As[buf], wm + a * 32, kg, lane);
#pragma unroll
        for (int c = 0; c < NBN; ++c) fb[set][c] = PB::fragment(Bs[buf], wn + c * 32, kg, lane);
    };
    typedef std::integral_constant<int, 0> I0;
    typedef std::integral_constant<int, 1> I1;
    auto block = [&](auto cur_c, auto load_c, const uint16_t *pa, const uint16_t *pb) __attribute__((always_inline)) {
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
            for (int a = 0; a < NBM; ++a) {
                if (a == NBM / 2 && kg == KG - 2) {
                    __builtin_amdgcn_sched_barrier(0);
                    PA::store(As[CUR ^ 1], ra[CUR ^ 1]);
                    PB::store(Bs[CUR ^ 1], rb[CUR ^ 1]);
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int c = 0; c < NBN; ++c)     // C^T = B^T A^T: lanes run along rows of C
                    acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[fs][c], fa[fs][a], acc[a][c], 0, 0, 0);
            }
            __builtin_amdgcn_s_setprio(0);
        }
    };
    // One tile.  On entry its panel 0 is in LDS buffer 0 with the first fragments read, panel 1 is
    // in staging set 1 (in flight), panel 2 in staging set 0 (in flight).
    auto run_tile = [&](const Loc &cur, const Loc &nxt) __attribute__((always_inline)) {
        const uint16_t *A = cur.A, *B = cur.B, *An = nxt.A, *Bn = nxt.B;
        uint16_t *C = cur.C;
#pragma unroll
        for (int a = 0; a < NBM; ++a)
#pragma unroll
            for (int c = 0; c < NBN; ++c)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[a][c][r] = 0.f;
        block(I0(), std::false_type(), A, B);                             // panel 2 was requested before the previous stores
        block(I1(), std::true_type(), A + 3 * panelA, B + 3 * panelB);
        const uint16_t *pa = A + 4 * panelA, *pb = B + 4 * panelB;
        for (int64_t kb = 2; kb < nkb; kb += 2) {
            if (kb + 2 == nkb) { pa = An; pb = Bn; }                      // the stream moves on to the next tile
            block(I0(), std::true_type(), pa, pb);
            pa += panelA; pb += panelB;
            block(I1(), std::true_type(), pa, pb);
            pa += panelA; pb += panelB;
        }
        gload(I0(), pa, pb);                                              // next tile's panel 2, ahead of the stores below
#pragma unroll
        for (int a = 0; a < NBM; ++a)
#pragma unroll
            for (int c = 0; c < NBN; ++c) {
                uint16_t *col = C + wm + a * 32 + (lane & 31) + (int64_t)(wn + c * 32 + 4 * (lane >> 5)) * g.ldc;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    uint16_t *dst = col + (8 * (r >> 2) + (r & 3)) * g.ldc;
                    float v = alpha * acc[a][c][r];
                    if (BETA) v += beta * sb_bf16_to_f32(*dst);
                    *dst = sb_f32_to_bf16(v);
                }
            }
    };

    Loc cur = locate(b, tile);
    {   // prime the stream with the first tile's panels 0, 1 and 2
        gload(I0(), cur.A, cur.B);
        gload(I1(), cur.A + panelA, cur.B + panelB);
        PA::store(As[0], ra[0]);
        PB::store(Bs[0], rb[0]);
        __syncthreads();
        read_frags(I0(), I0(), 0);
        gload(I0(), cur.A + 2 * panelA, cur.B + 2 * panelB);
    }
    // one tile and the step to the workgroup's next one; the last tile names itself as successor
    auto step = [&]() __attribute__((always_inline)) {
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

// Epilogue of a wave tile of NBM x NBN blocks whose accumulators hold C itself (MFMA with the A fragment
// first: lane l of block (a, c) holds column c*32 + l%32 and rows a*32 + 8g + 4(l/32) + q, slot 4g + q):
// alpha * acc rounded to bf16 goes through a wave-private LDS area of 64 columns x 32 rows (4 KB, [column][row],
// the 16-byte units of a column XORed with a function of the column: the 8-byte writes of a wave then hit each
// bank twice, the 16-byte reads once) and leaves in 16-byte stores, four lanes to a column: 64-byte runs that
// the next block row completes to whole lines.  A lane storing 2 bytes at a time needs eight times as many
// store instructions, and those, not the bytes, are what an epilogue costs (3.3 us per 256 x 256 tile).
// Only the wave itself touches the area, and LDS executes a wave's accesses in order: no barrier.
template <int NBM, int NBN>
__device__ __forceinline__ void store_wave_tile(uint16_t *area, const f32x16 (&acc)[NBM][NBN], uint16_t *Cw, int64_t ldc, float alpha, int lane)
{
    static_assert(NBN == 2, "the area holds 64 columns");
    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
    const int h = lane >> 5;
#pragma unroll
    for (int a = 0; a < NBM; ++a) {
#pragma unroll
        for (int c = 0; c < NBN; ++c) {
            const int col = c * 32 + (lane & 31);
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                u32x2 w;
                w[0] = (unsigned)sb_f32_to_bf16(alpha * acc[a][c][4 * g]) | ((unsigned)sb_f32_to_bf16(alpha * acc[a][c][4 * g + 1]) << 16);
                w[1] = (unsigned)sb_f32_to_bf16(alpha * acc[a][c][4 * g + 2]) | ((unsigned)sb_f32_to_bf16(alpha * acc[a][c][4 * g + 3]) << 16);
                *(u32x2 *)(area + col * 32 + ((g ^ ((col >> 2) & 3)) << 3) + h * 4) = w;
            }
        }
#pragma unroll
        for (int t = 0; t < NBN * 2; ++t) {
            const int u = lane + 64 * t, col = u >> 2, rq = u & 3;
            const u16x8 v = *(const u16x8 *)(area + col * 32 + ((rq ^ ((col >> 2) & 3)) << 3));
            *(u16x8u *)(Cw + a * 32 + rq * 8 + (int64_t)col * ldc) = v;
        }
    }
}

// LDS panel of the direct-to-LDS kernel for an operand whose 256 ROWS (m or n) are contiguous in memory: it is
// kept as it lies, [k][row], and transposed by the fragment read (ds_read_b64_tr_b16: in each group of 16 lanes,
// lanes 4r .. 4r+3 point at 16 consecutive rows of k-row r and lane j receives row j of the four k-rows, so two
// reads give a lane its 8 consecutive k).  A k-row is 512 bytes = 16 segments of 16 rows; segment s of k-row k
// sits at position s ^ 2 (k % 4), which puts the eight segments a half wave reads (two neighbouring ones at four
// consecutive k) on all banks.  Only whole 16-byte slots move, so the placement is free: the loads decide it.
struct PanelRows {
    static constexpr int ROWS = 256;
    // element offset inside the panel of (k, row), row a multiple of 4: slot of 16 rows, then the row inside it
    static __device__ __forceinline__ int at(int k, int row) { return k * ROWS + (((row >> 4) ^ (2 * (k & 3))) << 4) + (row & 15); }
    // what the 16-byte slot `slot16` of the panel holds: k and first row
    static __device__ __forceinline__ void source(int slot16, int &k, int &row)
    {
        k = slot16 >> 5;
        const int pos = slot16 & 31;                      // 16-byte position inside the k-row
        row = ((((pos >> 1) ^ (2 * (k & 3))) << 1) | (pos & 1)) << 3;
    }
    static __device__ __forceinline__ bf16x8 fragment(const uint16_t *lds, int row0, int ks, int lane)
    {
        typedef short s16x4 __attribute__((ext_vector_type(4)));
        typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
        const int i = lane & 15, g16 = lane >> 4;
        const int k = ks * 16 + 8 * (g16 >> 1) + (i >> 2);                   // this lane's address: k-row of its quad, +4 for the second read
        const int row = row0 + 16 * (g16 & 1) + 4 * (i & 3);
        const uint16_t *p = lds + at(k, row);
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)p);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + 4 * ROWS));     // (k + 4) % 4 == k % 4: same placement
        typedef short s16x8 __attribute__((ext_vector_type(8)));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    }
};

// Direct-to-LDS member of the streaming family: 256 x 256 tiles on eight waves of 128 x 64, both operands
// k-contiguous, 64 k per panel, two LDS stages of 64 KB.  The next panel travels from memory into the stage that
// the barrier has just freed while the current one is multiplied; no registers stage it, which leaves room for
// whole 128-byte lines per row (a 32-deep panel fetches half of each line and the other half a panel later,
// when the line has left the first-level cache) and removes the LDS store instructions with their register
// traffic.  On this chip a dense bf16 product with random operands runs against the power limit, not the
// issue rate (the same instruction stream is 1.25-1.35x faster on zeros), so bytes moved per flop count twice.
// Per panel and wave: four k-steps of 6 fragment reads and 8 MFMAs, two fragment sets; before the last k-step:
// wait for the panel in flight, barrier, request the panel after it, first fragments of the new stage.
// The swizzled [row][k] layout of a k-contiguous operand is produced by the choice of what each lane fetches:
// lane l of load j fills chunk slot 64 (8 j + wave) + l, i.e. row slot / 8, and fetches that row's k-chunk
// (slot % 8) ^ f(row).  An operand with m or n contiguous lands as [k][row] (PanelRows) and is transposed by its
// fragment reads: twice as many LDS instructions for that operand, nothing else.
template <bool BETA, bool A_KC, bool B_KC>
__global__ __launch_bounds__(512, 1) void sbgemm_bf16_dma_kernel(SbArgs g, int tiles_m, int tiles_n)
{
    constexpr int NBM = 4, NBN = 2, SBK = 64, WAVES_M = 2, WAVES_N = 4, KG = SBK / 16;
    constexpr int WM = 32 * NBM, WN = 32 * NBN, TM = WAVES_M * WM, TN = WAVES_N * WN, NT = 64 * WAVES_M * WAVES_N;
    typedef PanelBf16<true, TM, SBK, true, NT> P;            // layout and fragment reads (TM == TN)
    static_assert(TM == TN, "one panel type for both operands");
    constexpr int NLOAD = P::NVEC;                           // 16-byte loads per lane, operand and panel: 4
    constexpr int STAGE = 2 * P::LDS_SIZE;                   // elements per stage: A panel, B panel
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];      // [stage][A | B], then 4 KB per wave for the epilogue

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave % WAVES_M) * WM, wn = (wave / WAVES_M) * WN;
    const float alpha = (float)g.alpha, beta = (float)g.beta;
    const int64_t nkb = g.k / SBK;
    // leading dimension of a panel (row stride of a k-contiguous operand, k stride of the other kind) and the
    // element step from one panel to the next
    const int64_t ldA = A_KC ? g.rsA : g.csA, ldB = B_KC ? g.csB : g.rsB;
    const int64_t panelA = A_KC ? SBK : (int64_t)SBK * g.csA, panelB = B_KC ? SBK : (int64_t)SBK * g.rsB;

    const int64_t tiles = (int64_t)tiles_m * tiles_n;
    const int64_t total = tiles * g.batch0 * g.batch1;
    const int64_t nslots = (int64_t)gridDim.x / NXCD;           // the launcher makes gridDim.x a multiple of 8
    const int64_t xcd = blockIdx.x % NXCD, slot = blockIdx.x / NXCD;
    const int64_t q8 = total / NXCD, r8 = total % NXCD;
    const int64_t first = xcd * q8 + (xcd < r8 ? xcd : r8);
    const int64_t last = first + q8 + (xcd < r8 ? 1 : 0);
    int64_t logical = first + slot;
    if (logical >= last) return;

    // what this lane fetches: byte offsets from the panel's first element, per load; and where its wave's loads land
    unsigned offA[NLOAD], offB[NLOAD];
#pragma unroll
    for (int j = 0; j < NLOAD; ++j) {
        const int slot16 = 64 * (8 * j + wave) + lane;          // 16-byte slot inside the panel
        int rowk = slot16 / P::CPR, kk = P::swizzled(rowk, (slot16 % P::CPR) * 8);      // the swizzle is its own inverse
        int kr, rowr;
        PanelRows::source(slot16, kr, rowr);
        offA[j] = (unsigned)((A_KC ? (int64_t)rowk * ldA + kk : (int64_t)kr * ldA + rowr) * 2);
        offB[j] = (unsigned)((B_KC ? (int64_t)rowk * ldB + kk : (int64_t)kr * ldB + rowr) * 2);
    }
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) uint16_t *)lds;
    const unsigned land = __builtin_amdgcn_readfirstlane(lds0 + wave * 1024);           // + 8192 j, + P::LDS_SIZE * 2 for B, + STAGE * 2 per stage

    bf16x8 fa[2][NBM], fb[2][NBN];
    f32x16 acc[NBM][NBN];

    struct Loc { const uint16_t *A, *B; uint16_t *C; };
    auto locate = [&](int64_t b, int tile) __attribute__((always_inline)) {
        int64_t b0 = b, b1 = 0;
        if (g.batch1 != 1) { b1 = b / g.batch0; b0 = b - b1 * g.batch0; }
        const SbOff3 o1 = sb_level1(g, b1);
        const unsigned tn = (unsigned)tile / (unsigned)tiles_m, tm = (unsigned)tile - tn * (unsigned)tiles_m;
        const int64_t i0 = (int64_t)tm * TM, j0 = (int64_t)tn * TN;
        Loc l;
        l.A = (const uint16_t *)g.A + b0 * g.bsA[0] + o1.a + i0 * g.rsA;
        l.B = (const uint16_t *)g.B + b0 * g.bsB[0] + o1.b + j0 * g.csB;
        l.C = (uint16_t *)g.C + b0 * g.bsC[0] + o1.c + i0 + j0 * g.ldc;
        return l;
    };
    int64_t b = logical / tiles;
    int tile = (int)(logical - b * tiles);
    const int64_t dq = nslots / tiles;
    const int dr = (int)(nslots - dq * tiles);

    typedef std::integral_constant<int, 0> I0;
    typedef std::integral_constant<int, 1> I1;
    // request one panel (A rows at pa, B columns at pb) into stage ST
    auto request = [&](auto st_c, const uint16_t *pa, const uint16_t *pb) __attribute__((always_inline)) {
        constexpr int ST = decltype(st_c)::value;
#pragma unroll
        for (int j = 0; j < NLOAD; ++j) dma16(land + ST * STAGE * 2 + j * 8192, pa, offA[j]);
#pragma unroll
        for (int j = 0; j < NLOAD; ++j) dma16(land + ST * STAGE * 2 + P::LDS_SIZE * 2 + j * 8192, pb, offB[j]);
    };
    auto read_frags = [&](auto set_c, auto st_c, int kg) __attribute__((always_inline)) {
        constexpr int SET = decltype(set_c)::value, ST = decltype(st_c)::value;
        const uint16_t *As = lds + ST * STAGE, *Bs = As + P::LDS_SIZE;
#pragma unroll
        for (int a = 0; a < NBM; ++a) fa[SET][a] = A_KC ? P::fragment(As, wm + a * 32, kg, lane) : PanelRows::fragment(As, wm + a * 32, kg, lane);
#pragma unroll
        for (int c = 0; c < NBN; ++c) fb[SET][c] = B_KC ? P::fragment(Bs, wn + c * 32, kg, lane) : PanelRows::fragment(Bs, wn + c * 32, kg, lane);
    };
    auto mfmas = [&](auto set_c) __attribute__((always_inline)) {
        constexpr int SET = decltype(set_c)::value;
        __builtin_amdgcn_s_setprio(2);
#pragma unroll
        for (int a = 0; a < NBM; ++a)
#pragma unroll
            for (int c = 0; c < NBN; ++c)     // beta == 0: C itself (lanes along columns, slots along rows: the epilogue transposes in LDS);
                                              // else C^T = B^T A^T (lanes along rows: 2-byte stores straight from the accumulators)
                acc[a][c] = BETA ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[SET][c], fa[SET][a], acc[a][c], 0, 0, 0)
                                 : __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[SET][a], fb[SET][c], acc[a][c], 0, 0, 0);
        __builtin_amdgcn_s_setprio(0);
    };
    // One panel in stage ST.  On entry fragment set 0 holds (or is about to receive) its first k-step and the next
    // panel is in flight into the other stage; pa / pb: the panel after that one, requested once the barrier has
    // freed this stage.
    auto panel = [&](auto st_c, const uint16_t *pa, const uint16_t *pb) __attribute__((always_inline)) {
        constexpr int ST = decltype(st_c)::value;
        typedef std::integral_constant<int, ST> S;
        typedef std::integral_constant<int, ST ^ 1> SN;
        read_frags(I1(), S(), 1);
        mfmas(I0());
        read_frags(I0(), S(), 2);
        mfmas(I1());
        read_frags(I1(), S(), 3);
        mfmas(I0());
        __builtin_amdgcn_sched_barrier(0);
        dma_wait<0>();
        __syncthreads();
        request(S(), pa, pb);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(I0(), SN(), 0);
        mfmas(I1());
    };
    // One tile: its panel 0 is complete in stage 0 with the first fragments requested, panel 1 in flight into
    // stage 1; pa / pb point at panel 2.
    auto run_tile = [&](const Loc &cur, const Loc &nxt, const uint16_t *&pa, const uint16_t *&pb) __attribute__((always_inline)) {
#pragma unroll
        for (int a = 0; a < NBM; ++a)
#pragma unroll
            for (int c = 0; c < NBN; ++c)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[a][c][r] = 0.f;
        for (int64_t kb = 0; kb < nkb; kb += 2) {
            if (kb + 2 == nkb) { pa = nxt.A; pb = nxt.B; }                // panel kb + 2 is the next tile's first
            panel(I0(), pa, pb);
            pa += panelA; pb += panelB;
            panel(I1(), pa, pb);
            pa += panelA; pb += panelB;
        }
        uint16_t *C = cur.C;
        if (!BETA) {
            store_wave_tile<NBM, NBN>(lds + 2 * STAGE + wave * 2048, acc, C + wm + (int64_t)wn * g.ldc, g.ldc, alpha, lane);
            return;
        }
#pragma unroll
        for (int a = 0; a < NBM; ++a)
#pragma unroll
            for (int c = 0; c < NBN; ++c) {
                uint16_t *col = C + wm + a * 32 + (lane & 31) + (int64_t)(wn + c * 32 + 4 * (lane >> 5)) * g.ldc;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    uint16_t *dst = col + (8 * (r >> 2) + (r & 3)) * g.ldc;
                    float v = alpha * acc[a][c][r];
                    if (BETA) v += beta * sb_bf16_to_f32(*dst);
                    *dst = sb_f32_to_bf16(v);
                }
            }
    };

    Loc cur = locate(b, tile);
    const uint16_t *pa = cur.A + 2 * panelA, *pb = cur.B + 2 * panelB;
    request(I0(), cur.A, cur.B);
    request(I1(), cur.A + panelA, cur.B + panelB);
    dma_wait<2 * NLOAD>();                 // panel 0 has landed; panel 1 may still be under way
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

// whole tiles, an even number (>= 4) of k panels; either orientation of each operand
bool stream_applies(const SbArgs &a, int tile, int SBK)
{
    const bool a_ok = a.csA == 1 || a.rsA == 1, b_ok = a.rsB == 1 || a.csB == 1;
    return a_ok && b_ok && a.m % tile == 0 && a.n % tile == 0 && a.k % (2 * SBK) == 0 && a.k >= 4 * SBK;
}

// the streaming kernel for the orientation of the operands (k contiguous or rows contiguous, each)
template <bool BETA, int NBM, int NBN, int SBK, int WAVES_M, int WAVES_N, typename Launch>
hipError_t stream_by_layout(const SbArgs &a, Launch launch)
{
    const bool ak = a.csA == 1, bk = a.rsB == 1;
    if (ak && bk)  return launch(sbgemm_bf16_stream_kernel<BETA, NBM, NBN, SBK, WAVES_M, WAVES_N, true, true>);
    if (ak && !bk) return launch(sbgemm_bf16_stream_kernel<BETA, NBM, NBN, SBK, WAVES_M, WAVES_N, true, false>);
    if (!ak && bk) return launch(sbgemm_bf16_stream_kernel<BETA, NBM, NBN, SBK, WAVES_M, WAVES_N, false, true>);
    return launch(sbgemm_bf16_stream_kernel<BETA, NBM, NBN, SBK, WAVES_M, WAVES_N, false, false>);
}

template <typename K>
hipError_t launch_stream(K kernel, int tile, const SbArgs &a, hipStream_t stream, int nthreads = NTHREADS)
{
    const int64_t tiles_m = a.m / tile, tiles_n = a.n / tile;
    const int64_t total = tiles_m * tiles_n * a.batch0 * a.batch1;
    if (total <= 0) return hipSuccess;
    if (total >= (int64_t)1 << 31) return hipErrorInvalidConfiguration;
    int resident = 0;
    const hipError_t e = sb_resident_workgroups((const void *)kernel, nthreads, &resident);
    if (e != hipSuccess) return e;
    int64_t grid = total < resident ? total : resident;
    grid = (grid + NXCD - 1) / NXCD * NXCD;
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(nthreads), 0, stream, a, (int)tiles_m, (int)tiles_n);
    return hipGetLastError();
}

// the direct-to-LDS kernel: each operand k-contiguous or row-contiguous, an even number of 64-deep panels,
// offsets inside a panel (256 rows or 64 k-rows of the leading dimension) that fit the 32-bit lane offsets
bool dma_applies(const SbArgs &a)
{
    const int64_t most = (int64_t)1 << 22;
    const bool a_ok = a.csA == 1 || a.rsA == 1, b_ok = a.rsB == 1 || a.csB == 1;
    return a_ok && b_ok && a.k % 128 == 0 && a.rsA <= most && a.csA <= most && a.rsB <= most && a.csB <= most;
}

template <bool BETA, bool A_KC, bool B_KC>
hipError_t launch_dma(const SbArgs &a, hipStream_t stream)
{
    const int lds_bytes = 2 * 2 * 256 * 64 * 2 + 8 * 4096;  // two stages of an A and a B panel, the epilogue areas of eight waves
    auto kernel = sbgemm_bf16_dma_kernel<BETA, A_KC, B_KC>;
    static std::atomic<bool> configured[SB_MAX_DEVICES] = {};
    const int dev = sb_current_device();
    if (!configured[dev]) {
        const hipError_t e = hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        configured[dev] = true;
    }
    const int64_t tiles_m = a.m / 256, tiles_n = a.n / 256;
    const int64_t total = tiles_m * tiles_n * a.batch0 * a.batch1;
    if (total <= 0) return hipSuccess;
    if (total >= (int64_t)1 << 31) return hipErrorInvalidConfiguration;
    int resident = 0;                                       // one workgroup per compute unit (512 lanes of > 128 registers)
    const hipError_t e = sb_resident_workgroups((const void *)kernel, 512, &resident);
    if (e != hipSuccess) return e;
    int64_t grid = total < resident ? total : resident;
    grid = (grid + NXCD - 1) / NXCD * NXCD;
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(512), lds_bytes, stream, a, (int)tiles_m, (int)tiles_n);
    return hipGetLastError();
}

template <int WT>
hipError_t launch(const SbArgs &a, hipStream_t stream)
{
    constexpr int BM = 2 * WT, BN = 2 * WT;
    const int64_t tiles_m = (a.m + BM - 1) / BM, tiles_n = (a.n + BN - 1) / BN;
    const int64_t total = tiles_m * tiles_n * a.batch0 * a.batch1;
    if (total <= 0) return hipSuccess;
    if (total > sb_max_grid_x(NTHREADS)) return hipErrorInvalidConfiguration;     // sb_mfma_supports keeps such problems away
    const bool a_kc = (a.csA == 1), b_kc = (a.rsB == 1);
    // per operand (bit 0: A, bit 1: B): 16-byte vector loads; the hardware reads them at any
    // element-aligned address, so no leading dimension or offset has to be a multiple of 8
    const int vec_ok = 3;
    dim3 grid((unsigned)total), block(NTHREADS);
    const int tm = (int)tiles_m, tn = (int)tiles_n;
    if (a_kc && b_kc)        hipLaunchKernelGGL((sbgemm_mfma_bf16_kernel<true, true, WT>), grid, block, 0, stream, a, tm, tn, vec_ok);
    else if (a_kc && !b_kc)  hipLaunchKernelGGL((sbgemm_mfma_bf16_kernel<true, false, WT>), grid, block, 0, stream, a, tm, tn, vec_ok);
    else if (!a_kc && b_kc)  hipLaunchKernelGGL((sbgemm_mfma_bf16_kernel<false, true, WT>), grid, block, 0, stream, a, tm, tn, vec_ok);
    else                     hipLaunchKernelGGL((sbgemm_mfma_bf16_kernel<false, false, WT>), grid, block, 0, stream, a, tm, tn, vec_ok);
    return hipGetLastError();
}

}  // namespace

hipError_t sb_launch_mfma_bf16(const SbArgs &a, hipStream_t stream)
{
    // whole 128 x 128 tiles, both operands k-contiguous: the streaming kernel
    // (256 x 256 tiles when there are enough of them to fill the chip and k is long: measured 1.06-1.10x
    // over the 128 x 128 tiles at k = 2048-4096, 0.87x at k = 512, where a tile ends too soon)
    // (256 x 256 tiles on eight waves, 1.15-1.3x faster per flop, unless they would leave compute
    // units idle: few tiles, or a last round that is mostly empty)
    const int64_t batch = a.batch0 * a.batch1;
    if (stream_applies(a, 256, 32) && sb_tile_time((a.m / 256) * (a.n / 256) * batch, 4.0, 1.15) <=
                                          sb_tile_time(((a.m + 127) / 128) * ((a.n + 127) / 128) * batch, 1.0, 1.0)) {
        auto go = [&](auto kernel) { return launch_stream(kernel, 256, a, stream, 512); };
        if (dma_applies(a)) {
            const bool ak = a.csA == 1, bk = a.rsB == 1, b0 = a.beta == 0.0;
            if (ak && bk)  return b0 ? launch_dma<false, true, true>(a, stream) : launch_dma<true, true, true>(a, stream);
            if (ak && !bk) return b0 ? launch_dma<false, true, false>(a, stream) : launch_dma<true, true, false>(a, stream);
            if (!ak && bk) return b0 ? launch_dma<false, false, true>(a, stream) : launch_dma<true, false, true>(a, stream);
            return b0 ? launch_dma<false, false, false>(a, stream) : launch_dma<true, false, false>(a, stream);
        }
        if (a.beta == 0.0) return stream_by_layout<false, 4, 2, 32, 2, 4>(a, go);
        return stream_by_layout<true, 4, 2, 32, 2, 4>(a, go);
    }
    if (stream_applies(a, 128, 64)) {
        auto go = [&](auto kernel) { return launch_stream(kernel, 128, a, stream); };
        if (a.beta == 0.0) return stream_by_layout<false, 2, 2, 64, 2, 2>(a, go);
        return stream_by_layout<true, 2, 2, 64, 2, 2>(a, go);
    }
    // small matrices per batch: 64x64 tiles waste less and give more workgroups
    if (a.m <= 64 || a.n <= 64) return launch<32>(a, stream);
    return launch<64>(a, stream);
}
