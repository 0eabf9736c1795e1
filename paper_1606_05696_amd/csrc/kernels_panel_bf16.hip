// Whole-K panel-grid kernel for bf16 products with a short inner extent (k <= 128).
//
// With k this short the product is bound by writing C, not by the matrix cores: every operand
// panel (64 rows x k, k x 64 columns) fits LDS whole, and the job is to keep the stores flowing.
// The kernel sees C as a GRID of 64 x 64 blocks C[r][c] = Apanel[r] * Bpanel[c] in which the row
// panel r does not depend on c and the column panel c does not depend on r.  A row panel is a run of
// up to 64 rows of one op(A) matrix, a column panel a run of up to 64 columns of one op(B) matrix;
// the panel index of a side counts, mixed radix, the 64-wide pieces of the flat extent and every
// batch level that moves this side's operand only.  That one picture holds
//   - the nested batch  C_m[p]n[q] = A_m[p]k B_kn[q]   (section III-F, Listing 2): rows = p, columns = q,
//   - its flattened GEMM  C_(mp)(nq) = A_(mp)k B_k(nq)  (priority 1 of section IV-D): rows and columns
//     are 64-wide pieces of the flat extents,
//   - the partly flattened forms  C_(mp)n[q]  and  C_m[p](nq),
// so all evaluations of such a contraction run through the same code at the same speed: the batch
// loops are part of the tiling (what section III-D expects of a StridedBatchedGemm implementation).
// Batch levels that move both operands (or neither) are an outer index z: independent grids.
//
// A workgroup of eight waves takes a block of 4 x 4 panels (256 x 256 outputs): 4 + 4 panels are
// fetched for 16 small products, so the nest gets the operand reuse of a tiled GEMM although
// nothing is flattened or copied.  Wave w owns row panel w % 4 and the left or right 32 columns of
// every column panel; its A fragments (64 rows x k) stay in registers for all four column panels,
// so a product reads only its B fragments from LDS (the matrix cores would otherwise wait for LDS:
// 32 KB of fragment reads per 64 x 64 x 128 product against 1024 matrix-core cycles).
// All 16 operand loads of a lane are issued at once; the A panels are handed to LDS first, then
// the first column panel, and the other three while the first product runs.  Results leave through a
// per-wave staging area in LDS (the A region, free once the fragments are in registers) as whole
// 128-byte lines of C; a wave's stores drain while the next product runs, and no workgroup-wide
// barrier separates the products.
// Every panel is kept [row][k] in LDS, whatever the operand's orientation in memory, so that an
// MFMA operand is ONE 16-byte LDS read.  An operand with m (or n) contiguous in memory is transposed
// on the way in: a lane loads an 8 x 8 block (8 vectors of 8 rows, one per k), transposes it in
// registers and writes 8 vectors of 8 k; the 16-byte chunk index of such a panel is XORed with
// (row / 8) % 8 on the write and on the read side, which keeps those writes off the same banks.
// Vector accesses need no alignment beyond the element's (the hardware reads and writes 16 bytes
// at any element address).  RAGGED instantiations handle extents that are not whole vectors with
// guarded element accesses; the others keep every load unconditional so that the hand-over to LDS
// can wait for exactly the loads it needs.
//
// A second member further down takes the whole-panel k = 128 problems: blocks of 2 x 8 panels whose operands
// travel straight into LDS (sbgemm_panelgrid_wide_bf16_kernel); this one serves every other shape.
#include "sb_device.h"
#include "sb_internal.h"

#include <atomic>
#include <type_traits>

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short u16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4u __attribute__((ext_vector_type(4), aligned(2)));      // global access at any element address

// how a result vector goes to C (a 16-byte store at any element address)
// C is written once and not read again by this kernel: non-temporal stores let the lines stream
// through the L2 instead of waiting there for the write-back at the end of the kernel
#ifndef SB_PANEL_STORE
#define SB_PANEL_STORE(ptr, value) __builtin_nontemporal_store((value), (ptr))
#endif

constexpr int TM = 64, KMAX = 128;
constexpr int LD_KC = KMAX + 8;           // [row][k] layout, rows padded by 16 bytes
constexpr int PANEL = TM * LD_KC;         // elements of one panel in LDS
constexpr int BR = 4, BC = 4;             // panels per workgroup block
constexpr int NT = 512;                   // eight waves
constexpr int SPITCH = 68;                // staged column: 64 rows + 8 bytes
constexpr int LDS_ELEMS = (BR + BC) * PANEL;
static_assert(8 * 2 * 32 * SPITCH <= BR * PANEL, "two staging areas for each of the eight waves fit the A region");

// Division of a number below 2^31 by a divisor fixed on the host: one multiply-high, one add, one
// shift (Granlund and Montgomery's round-up method; with n < 2^31 the add cannot overflow).  The
// decode of a workgroup's block would otherwise spend a microsecond in emulated integer divisions
// before the first load is issued.
struct FastDiv {
    uint32_t mul, shift;
};
__device__ __forceinline__ unsigned fdiv(unsigned n, FastDiv d) { return (__umulhi(n, d.mul) + n) >> d.shift; }

// One side of the panel grid: rows of C (operand A) or columns of C (operand B).
struct Side {
    int32_t nf, n1, n2;        // 64-wide pieces of the flat extent; counts of up to two batch levels of this side
    FastDiv dnf, dn1;
    int32_t full, last;        // rows (columns) in a piece of the flat extent: every one but the last / the last
    int64_t sf, s1, s2;        // element strides in the operand: between pieces, per batch level
    int64_t cf, c1, c2;        // the same in C
    uint32_t ld;               // operand: stride between rows (k contiguous) or between k (rows contiguous), below 2^31
};

struct PanelArgs {
    const uint16_t *A, *B;
    uint16_t *C;
    Side row, col;
    int32_t R, Cn;             // row panels, column panels
    int32_t nrb, ncb;          // blocks of 4 along each side
    int32_t nsc;               // super-tiles (4 x 8 blocks) along the columns
    int32_t per_z;             // block slots per outer index (super-tiles are padded)
    int32_t z0, z1;            // outer batch levels
    FastDiv dper_z, dnsc, dz0;
    int64_t zA[2], zB[2], zC[2];
    int64_t ldc;
    int32_t k;
    float alpha, beta;
};

struct Loc {
    int64_t off, offC;         // element offsets of the panel in its operand and in C
    int32_t ext;               // rows (columns) of the panel
};

// panel idx of a side (the last valid one if idx is beyond `count`).  For an index that differs from
// wave to wave: indexing the arrays below with it would move them from registers to scratch memory.
__device__ __forceinline__ Loc locate1(const Side &s, int idx, int count)
{
    if (idx >= count) idx = count - 1;
    const unsigned t = fdiv((unsigned)idx, s.dnf), f = (unsigned)idx - t * (unsigned)s.nf;
    const unsigned l2 = fdiv(t, s.dn1), l1 = t - l2 * (unsigned)s.n1;
    Loc r;
    r.off = (int64_t)f * s.sf + (int64_t)l1 * s.s1 + (int64_t)l2 * s.s2;
    r.offC = (int64_t)f * s.cf + (int64_t)l1 * s.c1 + (int64_t)l2 * s.c2;
    r.ext = (int)f == s.nf - 1 ? s.last : s.full;
    return r;
}

// the N consecutive panels idx0 .. idx0+N-1 of a side; beyond `count` the last valid one is repeated
// (its data is loaded again and never stored).  One decode, then a mixed-radix odometer.
template <int N>
__device__ __forceinline__ void locate_run(const Side &s, int idx0, int count, Loc (&out)[N])
{
    const unsigned t = fdiv((unsigned)idx0, s.dnf);
    unsigned f = (unsigned)idx0 - t * (unsigned)s.nf;
    unsigned l2 = fdiv(t, s.dn1), l1 = t - l2 * (unsigned)s.n1;
    out[0].off = (int64_t)f * s.sf + (int64_t)l1 * s.s1 + (int64_t)l2 * s.s2;
    out[0].offC = (int64_t)f * s.cf + (int64_t)l1 * s.c1 + (int64_t)l2 * s.c2;
    out[0].ext = (int)f == s.nf - 1 ? s.last : s.full;
#pragma unroll
    for (int i = 1; i < N; ++i) {
        out[i] = out[i - 1];
        if (idx0 + i < count) {
            if (++f < (unsigned)s.nf) {          // the next piece of the same matrix: two additions
                out[i].off += s.sf;
                out[i].offC += s.cf;
            } else {                             // first piece of the next batch entry
                f = 0;
                if (++l1 == (unsigned)s.n1) { l1 = 0; ++l2; }
                out[i].off = (int64_t)l1 * s.s1 + (int64_t)l2 * s.s2;
                out[i].offC = (int64_t)l1 * s.c1 + (int64_t)l2 * s.c2;
            }
            out[i].ext = (int)f == s.nf - 1 ? s.last : s.full;
        }
    }
}

// The four panels of one side on their way from memory to LDS, spread over all 512 lanes: load() only
// issues the global loads, store<P0, P1>() hands the panels P0 .. P1-1 to LDS in [row][k] form.
//   KC (k contiguous in memory): 4 x 1024 vectors, straight copy; vector i of a lane belongs to panel i / 2.
//   otherwise (rows contiguous): one 8 x 8 block per lane (8 vectors of 8 rows), transposed in registers;
//     a lane's block belongs to panel tid / 128, so the four panels can only be stored together.
template <bool KC, bool RAGGED>
struct FourPanels {
    u32x4 v[8];

    static __device__ __forceinline__ u32x4 guarded(const uint16_t *src, int n_ok)      // first n_ok elements, zeros after
    {
        uint16_t e[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) e[q] = q < n_ok ? src[q] : (uint16_t)0;
        u32x4 w;
#pragma unroll
        for (int c = 0; c < 4; ++c) w[c] = (unsigned)e[2 * c] | ((unsigned)e[2 * c + 1] << 16);
        return w;
    }

    // loc: the four panels; mine: the panel of this lane's 8 x 8 block (rows-contiguous operands).
    // Panels P0 .. P1-1 (rows-contiguous operands: all four together, with P0 == 0).
    template <int P0, int P1>
    __device__ __forceinline__ void load(const uint16_t *X, const Loc (&loc)[4], const Loc &mine, uint32_t ld, int kk)
    {
        const int tid = (int)threadIdx.x;
        if (KC) {
#pragma unroll
            for (int i = 2 * P0; i < 2 * P1; ++i) {
                const int panel = i / 2, f = tid + NT * (i % 2);
                const int row = f / (KMAX / 8), k = (f % (KMAX / 8)) * 8;
                const uint16_t *base = X + loc[panel].off;
                if (RAGGED) {
                    const int n_ok = row < loc[panel].ext ? kk - k : 0;
                    if (n_ok >= 8) v[i] = *(const u32x4u *)(base + (uint64_t)((uint32_t)row * (uint64_t)ld + k));
                    else if (n_ok > 0) v[i] = guarded(base + (uint64_t)((uint32_t)row * (uint64_t)ld + k), n_ok);
                    else v[i] = u32x4{0, 0, 0, 0};
                } else {            // a vector outside the panel reads the panel's first one instead; store() drops it
                    const bool inside = row < loc[panel].ext && k < kk;
                    v[i] = *(const u32x4u *)(base + (inside ? (uint64_t)((uint32_t)row * (uint64_t)ld + k) : 0));
                }
            }
        } else if (P0 == 0) {
            const int blk = tid % 128;
            const int rg = blk % 8, kg = blk / 8;                  // rows 8 rg .. +7, k 8 kg .. +7
            const uint16_t *base = X + mine.off;
            const int ext = mine.ext;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int k = kg * 8 + i;
                if (RAGGED) {
                    const int n_ok = k < kk ? ext - rg * 8 : 0;
                    if (n_ok >= 8) v[i] = *(const u32x4u *)(base + (uint64_t)((uint32_t)k * (uint64_t)ld + rg * 8));
                    else if (n_ok > 0) v[i] = guarded(base + (uint64_t)((uint32_t)k * (uint64_t)ld + rg * 8), n_ok);
                    else v[i] = u32x4{0, 0, 0, 0};
                } else {
                    const bool inside = rg * 8 < ext && k < kk;
                    v[i] = *(const u32x4u *)(base + (inside ? (uint64_t)((uint32_t)k * (uint64_t)ld + rg * 8) : 0));
                }
            }
        }
    }

    // vectors outside the matrix become zeros here (not after the load, which would wait for it)
    template <int P0, int P1>
    __device__ __forceinline__ void store(uint16_t *lds, const Loc (&loc)[4], const Loc &mine, int kk) const
    {
        const int tid = (int)threadIdx.x;
        const u32x4 z = {0, 0, 0, 0};
        if (KC) {
#pragma unroll
            for (int i = 2 * P0; i < 2 * P1; ++i) {
                const int panel = i / 2, f = tid + NT * (i % 2);
                const int row = f / (KMAX / 8), k = (f % (KMAX / 8)) * 8;
                const bool inside = RAGGED || (row < loc[panel].ext && k < kk);      // RAGGED: load() already put the zeros in
                *(u32x4 *)(lds + panel * PANEL + row * LD_KC + k) = inside ? v[i] : z;
            }
        } else if (P0 == 0) {               // transposed in registers: row 8 rg + j gets its 8 k as 4 words
            const int panel = tid / 128, blk = tid % 128;
            const int rg = blk % 8, kg = blk / 8;
            const int ext = mine.ext;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                u32x4 w;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const bool in_lo = RAGGED || (rg * 8 < ext && kg * 8 + 2 * c < kk);
                    const bool in_hi = RAGGED || (rg * 8 < ext && kg * 8 + 2 * c + 1 < kk);
                    const unsigned lo = in_lo ? v[2 * c][j / 2] : 0u, hi = in_hi ? v[2 * c + 1][j / 2] : 0u;
                    w[c] = (j % 2 == 0) ? ((lo & 0xffffu) | (hi << 16)) : ((lo >> 16) | (hi & 0xffff0000u));
                }
                *(u32x4 *)(lds + panel * PANEL + (rg * 8 + j) * LD_KC + ((kg ^ rg) * 8)) = w;
            }
        }
    }
};

// MFMA operand of the 32 rows starting at row0 for k-step ks; SWZ: the panel was written with the chunk swizzle
template <bool SWZ>
__device__ __forceinline__ bf16x8 panel_fragment(const uint16_t *lds, int row0, int ks, int lane)
{
    const int row = row0 + (lane & 31);
    int chunk = ks * 2 + (lane >> 5);
    if (SWZ) chunk ^= (row >> 3) & 7;
    return __builtin_bit_cast(bf16x8, *(const u16x8 *)(lds + row * LD_KC + chunk * 8));
}

template <bool A_KC, bool B_KC, int KS, bool RAGGED>
__global__ __launch_bounds__(NT, 1) void sbgemm_panelgrid_bf16_kernel(PanelArgs g)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];      // [A0 .. A3 | B0 .. B3]; the A region becomes the staging area
    uint16_t *ldsA = lds, *ldsB = lds + BR * PANEL;
    const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // Workgroup -> block.  The hardware deals consecutive workgroup ids to the 8 XCDs in turn; renumber
    // so that each XCD owns a contiguous range of slots, and order the slots in super-tiles of 4 x 8
    // blocks so that such a range is a compact rectangle of the grid: an XCD's L2 then holds few
    // different panels (16 row and 32 column panels per super-tile).
    const unsigned total = gridDim.x, bid = blockIdx.x;
    const unsigned q8 = total >> 3, r8 = total & 7, xcd = bid & 7, slot = bid >> 3;
    const unsigned logical = xcd * q8 + (xcd < r8 ? xcd : r8) + slot;
    const unsigned z = fdiv(logical, g.dper_z), within = logical - z * (unsigned)g.per_z;
    const unsigned stile = within >> 5, in = within & 31;
    const unsigned srow = fdiv(stile, g.dnsc), scol = stile - srow * (unsigned)g.nsc;
    const int rb = (int)(srow * 4 + (in & 3)), cb = (int)(scol * 8 + (in >> 2));
    if (rb >= g.nrb || cb >= g.ncb) return;                 // padding slot of a ragged super-tile (whole workgroup)
    const unsigned zi1 = fdiv(z, g.dz0), zi0 = z - zi1 * (unsigned)g.z0;
    const int kk = g.k;

    // the loads go out as early as possible: row side, its loads, column side, its loads
    Loc rl[4], cl[4];
    Loc ra = {0, 0, 0}, ca = {0, 0, 0};          // rows-contiguous operands: the panel this lane's 8 x 8 block belongs to
    FourPanels<A_KC, RAGGED> pa;
    FourPanels<B_KC, RAGGED> pb;
    locate_run<4>(g.row, rb * BR, g.R, rl);
    if (!A_KC) ra = locate1(g.row, rb * BR + tid / 128, g.R);
    pa.template load<0, 4>(g.A + (int64_t)zi0 * g.zA[0] + (int64_t)zi1 * g.zA[1], rl, ra, g.row.ld, kk);
    locate_run<4>(g.col, cb * BC, g.Cn, cl);
    if (!B_KC) ca = locate1(g.col, cb * BC + tid / 128, g.Cn);
    // only the first column panel for now: the other three would queue ahead of slower waves' A loads
    const uint16_t *Bz = g.B + (int64_t)zi0 * g.zB[0] + (int64_t)zi1 * g.zB[1];
    pb.template load<0, 1>(Bz, cl, ca, g.col.ld, kk);

    // wave w: row panel w % 4, columns 32 (w / 4) .. +31 of every column panel
    const int pi = wave & 3, half = wave >> 2;
    const float alpha = g.alpha, beta = g.beta;
    const bool row_live = rb * BR + pi < g.R;
    const Loc my_row = locate1(g.row, rb * BR + pi, g.R);
    const int rows = my_row.ext;
    uint16_t *Crow = g.C + (int64_t)zi0 * g.zC[0] + (int64_t)zi1 * g.zC[1] + my_row.offC;
    uint16_t *st = ldsA + wave * (2 * 32 * SPITCH);       // two staging areas of 32 columns each

    pa.template store<0, 4>(ldsA, rl, ra, kk);
    pb.template store<0, 1>(ldsB, cl, ca, kk);
    pb.template load<1, 4>(Bz, cl, ca, g.col.ld, kk);
    __syncthreads();             // the row panels and the first column panel are in LDS
    bf16x8 fa[2][KS];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) fa[a][ks] = panel_fragment<!A_KC>(ldsA + pi * PANEL, a * 32, ks, lane);

    // result register r of lane l of an MFMA: row 8 (r/4) + 4 (l/32) + r%4, column l%32 of the 32 x 32 block
    auto clear = [&](f32x16 (&acc)[2]) __attribute__((always_inline)) {
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][r] = 0.f;
    };
    auto read_b = [&](bf16x8 (&fb)[KS], int s) __attribute__((always_inline)) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) fb[ks] = panel_fragment<!B_KC>(ldsB + s * PANEL, half * 32, ks, lane);
    };
    auto mfma_step = [&](f32x16 (&acc)[2], const bf16x8 (&fb)[KS], int ks) __attribute__((always_inline)) {
#pragma unroll
        for (int a = 0; a < 2; ++a) acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a][ks], fb[ks], acc[a], 0, 0, 0);
    };
    // One eighth of the finished product s (4 rows x 32 columns per half wave) scaled, rounded to bf16
    // and parked in the wave's staging area s % 2.  WITH_BETA: plus beta times the old C.
    auto stage_part = [&](const f32x16 (&acc)[2], int s, int part, auto with_beta) __attribute__((always_inline)) {
        const int a = part >> 2, g4 = part & 3, j = lane & 31;
        const int i0 = a * 32 + 8 * g4 + 4 * (lane >> 5);
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = alpha * acc[a][4 * g4 + e];
        if (decltype(with_beta)::value) {
            const bool live = row_live && cb * BC + s < g.Cn;
            if (live && j < cl[s].ext - half * 32) {
                const uint16_t *old = Crow + cl[s].offC + (int64_t)(half * 32 + j) * g.ldc + i0;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (i0 + e < rows) v[e] += beta * sb_bf16_to_f32(old[e]);
            }
        }
        u16x4 pk;
#pragma unroll
        for (int e = 0; e < 4; ++e) pk[e] = sb_f32_to_bf16(v[e]);
        *(u16x4 *)(st + (s & 1) * (32 * SPITCH) + j * SPITCH + i0) = pk;
    };
    // A quarter (8 columns) of the staged 64 x 32 block s goes to C as whole 128-byte lines.  The wave's
    // own LDS accesses execute in order, so the staged values are there; the fences at the call sites
    // keep the compiler from moving the reads above the writes.
    auto write_quarter = [&](int s, int t) __attribute__((always_inline)) {
        const bool live = row_live && cb * BC + s < g.Cn;
        const int cols = cl[s].ext - half * 32;              // columns of this wave's half that exist
        uint16_t *Cq = Crow + cl[s].offC + (int64_t)(half * 32) * g.ldc;
        const uint16_t *sb = st + (s & 1) * (32 * SPITCH);
        const int seg = 8 * (lane & 7), jj = 8 * t + (lane >> 3);
        const u16x4 lo = *(const u16x4 *)(sb + jj * SPITCH + seg);
        const u16x4 hi = *(const u16x4 *)(sb + jj * SPITCH + seg + 4);
        if (live && jj < cols) {
            uint16_t *dst = Cq + (int64_t)jj * g.ldc + seg;
            if (!RAGGED || seg + 8 <= rows) {
                if (seg < rows) {
                    u32x4 o;
                    o[0] = (unsigned)lo[0] | ((unsigned)lo[1] << 16);
                    o[1] = (unsigned)lo[2] | ((unsigned)lo[3] << 16);
                    o[2] = (unsigned)hi[0] | ((unsigned)hi[1] << 16);
                    o[3] = (unsigned)hi[2] | ((unsigned)hi[3] << 16);
                    SB_PANEL_STORE((u32x4u *)dst, o);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (seg + e < rows) dst[e] = lo[e];
                    if (seg + 4 + e < rows) dst[4 + e] = hi[e];
                }
            }
        }
    };
    auto wave_fence = [&]() __attribute__((always_inline)) {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };
    auto write_block = [&](int s) __attribute__((always_inline)) {
        wave_fence();
#pragma unroll
        for (int t = 0; t < 4; ++t) write_quarter(s, t);
        wave_fence();
    };
    const int nsteps = g.Cn - cb * BC < BC ? g.Cn - cb * BC : BC;       // column panels of this block (workgroup-uniform)
    // beta == 0: three products are in flight per wave.  In program order every pair of MFMAs of product
    // s+1 is followed by an eighth of the rounding and staging of product s and, every other time, by a
    // quarter of the stores of product s-1 (two staging areas alternate), so the matrix core, the vector
    // ALU, LDS and the store path work side by side instead of one after the other.
    // fb holds the B fragments of product s+1 on entry; each one is replaced by its successor of
    // product s+2 as soon as its MFMAs are issued, so no product starts by waiting for LDS.
    bf16x8 fb[KS];
    auto pipe_loop = [&](const f32x16 (&done)[2], f32x16 (&next)[2], int s, auto refill) __attribute__((always_inline)) {
        clear(next);
#pragma unroll
        for (int part = 0; part < 8; ++part) {
            if (part < KS) {
                mfma_step(next, fb, part);
                if (decltype(refill)::value) fb[part] = panel_fragment<!B_KC>(ldsB + (s + 2) * PANEL, half * 32, part, lane);
            }
            stage_part(done, s, part, std::false_type());
            if (s > 0 && (part & 1)) write_quarter(s - 1, part >> 1);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    auto pipelined = [&](const f32x16 (&done)[2], f32x16 (&next)[2], int s) __attribute__((always_inline)) {
        wave_fence();
        if (s + 2 < nsteps) {
            pipe_loop(done, next, s, std::true_type());
        } else if (s + 1 < nsteps) {
            pipe_loop(done, next, s, std::false_type());
        } else {
#pragma unroll
            for (int part = 0; part < 8; ++part) {
                stage_part(done, s, part, std::false_type());
                if (s > 0 && (part & 1)) write_quarter(s - 1, part >> 1);
            }
        }
    };

    f32x16 acc0[2], acc1[2];
    read_b(fb, 0);
    clear(acc0);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) mfma_step(acc0, fb, ks);
    pb.template store<1, 4>(ldsB, cl, ca, kk);  // the other three column panels, while the matrix cores run
    __syncthreads();             // they are in LDS, and every wave holds its A fragments: the A region is free for staging
    if (nsteps > 1) read_b(fb, 1);
    // written out: s is a constant in each call, so cl[] stays in registers
    if (beta == 0.f) {
        pipelined(acc0, acc1, 0);
        if (nsteps > 1) pipelined(acc1, acc0, 1);
        if (nsteps > 2) pipelined(acc0, acc1, 2);
        if (nsteps > 3) pipelined(acc1, acc0, 3);
        if (nsteps == 1) write_block(0);
        else if (nsteps == 2) write_block(1);
        else if (nsteps == 3) write_block(2);
        else write_block(3);
    } else {                     // beta != 0 reads C as well: one product after the other
#pragma unroll
        for (int s = 0; s < BC; ++s) {
            if (s < nsteps) {
                if (s > 0) {
                    if (s > 1) read_b(fb, s);                // product 1's fragments were requested above
                    clear(acc0);
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) mfma_step(acc0, fb, ks);
                }
#pragma unroll
                for (int part = 0; part < 8; ++part) stage_part(acc0, s, part, std::true_type());
                write_block(s);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Wide-block member: a workgroup takes 2 x 8 panels, and the operands travel straight into LDS.
//
// A compute unit that runs ONE block pays its whole start-up chain (launch, arguments, fetch, first
// product) before the first line of C leaves, and the stores, which bound the kernel (a step of 16 KB per
// compute unit takes 0.55-0.6 us whatever else happens: 7-7.5 TB/s over the chip), cannot start earlier
// than that.  So what the first product needs is small and everything else arrives behind it: two row panels
// and ONE column panel (48 KB instead of the 80 KB of a 4 x 4 block), after which a product (2 row panels
// x 1 column panel) follows every column panel as it lands.  Loads are global_load_lds_dwordx4 (no staging
// registers, no LDS store instructions, no register transposition), issued in the order of need, the
// first four column panels during start-up and one more behind each product's stores.  Vector-memory
// operations of a wave complete in issue order, so "column panel s+1 has landed" is a count of the
// operations the wave has issued after that panel's loads (wide_pending): younger loads plus two stores
// per finished product.
// Wave w owns row panel w % 2 and 16 of the 64 columns of every column panel (v_mfma_f32_16x16x32_bf16,
// lanes along the columns, four consecutive rows per lane); its A fragments (64 rows x 128 k) stay in
// registers, a product reads 4 KB of B fragments.  Per step: product s is rounded into the wave's staging
// area and leaves as whole 128-byte lines (non-temporal); then wait + barrier (panel s+1 is there), its B
// fragments, and the 16 MFMAs of product s+1.
// Panels are unpadded (ten of them fill the 160 KB), so conflicts are avoided by placement, which costs
// nothing because each lane chooses what it fetches into its linear 16-byte LDS slot:
//   k contiguous in memory:  [row][k], the 16-byte chunk c of row r at position c ^ (r % 16);
//   rows contiguous:         [k][row], kept as it lies and transposed by the fragment read
//                            (ds_read_b64_tr_b16), the 16-row segment s of k-row k at position
//                            s ^ (bit 1 of k | bit 3 of k << 1): the eight segments a half wave reads
//                            (four consecutive k at two k-groups) then lie on all banks.
// Taken when k == 128, beta == 0, every panel is whole, the grid is made of whole blocks and all
// addresses are 16-byte aligned; everything else runs the 4 x 4 kernel above.
constexpr int WR = 2, WC = 8;
constexpr int WPANEL = TM * KMAX;                    // elements of an unpadded panel (16 KB)
constexpr int WLDS_ELEMS = (WR + WC) * WPANEL;       // 160 KB
constexpr int WSTAGE = 16 * TM;                      // a staged product of a wave: 16 columns x 64 rows (2 KB)
static_assert(8 * 2 * WSTAGE <= WR * WPANEL, "two staging areas for each of the eight waves fit the A region");

typedef float f32x4 __attribute__((ext_vector_type(4)));

// Column panels 0 .. WAHEAD-1 are requested before the first product, panel s + WAHEAD in step s.
constexpr int WAHEAD = 4;
// Vector-memory operations a wave has issued after the two loads of column panel s+1 when step s waits for
// that panel.  A wave's sequence: the row panels, column panels 0 .. WAHEAD-1, then per step t the two stores
// of product t followed by the loads of panel t + WAHEAD (if there is one); step s waits at its end.
constexpr int wide_pending(int s)
{
    int n = 0;
    bool seen = false;
    for (int p = 0; p < WAHEAD; ++p) {
        if (seen) n += 2;
        if (p == s + 1) seen = true;
    }
    for (int t = 0; t <= s; ++t) {
        if (seen) n += 2;                                       // stores of product t
        if (t + WAHEAD < WC) {
            if (seen) n += 2;
            if (t + WAHEAD == s + 1) seen = true;
        }
    }
    return n;
}
static_assert(WAHEAD != 4 || (wide_pending(0) == 8 && wide_pending(1) == 10 && wide_pending(2) == 12 && wide_pending(3) == 12 &&
                              wide_pending(4) == 10 && wide_pending(5) == 8 && wide_pending(6) == 6), "hand count for four panels ahead");

// what the 16-byte LDS slot `slot16` of a panel holds, as an element offset into the operand (ld: elements
// between rows of a k-contiguous operand, between k of a row-contiguous one)
template <bool KC>
__device__ __forceinline__ unsigned wide_source(int slot16, unsigned ld)
{
    if (KC) {
        const int row = slot16 >> 4, chunk = (slot16 & 15) ^ (row & 15);
        return (unsigned)row * ld + (unsigned)chunk * 8;
    }
    const int k = slot16 >> 3, pos = slot16 & 7;
    const int f = ((k >> 1) & 1) | (((k >> 3) & 1) << 1);
    const int row = ((((pos >> 1) ^ f) << 1) | (pos & 1)) << 3;
    return (unsigned)k * ld + (unsigned)row;
}

// MFMA operand (16x16x32: lane l holds row row0 + l % 16, k = 32 ks + 8 (l / 16) .. + 7) of a panel
template <bool KC>
__device__ __forceinline__ bf16x8 wide_fragment(const uint16_t *panel, int row0, int ks, int lane)
{
    if (KC) {
        const int row = row0 + (lane & 15), chunk = (4 * ks + (lane >> 4)) ^ (row & 15);
        return __builtin_bit_cast(bf16x8, *(const u16x8 *)(panel + row * KMAX + chunk * 8));
    }
    // in each group of 16 lanes, lanes 4r .. 4r+3 point at 16 consecutive rows of k-row r and lane j receives
    // row j of the four k-rows: two reads give a lane its 8 consecutive k
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const int i = lane & 15, g16 = lane >> 4;
    const int k = ks * 32 + 8 * g16 + (i >> 2);
    const int f = ((k >> 1) & 1) | (((k >> 3) & 1) << 1);
    const uint16_t *p = panel + k * TM + (((row0 >> 4) ^ f) << 4) + 4 * (i & 3);
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)p);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + 4 * TM));      // k + 4: same placement
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// PADDED: the launch holds padding slots (super-tiles at the edge of the block grid that are not full).  Without
// them nothing branches before the loads, so all kernel arguments are fetched in one round trip (a scalar load
// of arguments takes some 0.3 us here, and the early exit would put a second one behind the first).
template <bool A_KC, bool B_KC, bool PADDED>
__global__ __launch_bounds__(NT, 1) void sbgemm_panelgrid_wide_bf16_kernel(PanelArgs g)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];      // [A0 A1 | B0 .. B7]; the A region becomes the staging area
    uint16_t *ldsA = lds, *ldsB = lds + WR * WPANEL;
    const int tid = (int)threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // Workgroup -> block: as above, with super-tiles of 8 x 4 blocks (again 16 row and 32 column panels).
    const unsigned total = gridDim.x, bid = blockIdx.x;
    const unsigned q8 = total >> 3, r8 = total & 7, xcd = bid & 7, slot = bid >> 3;
    const unsigned logical = xcd * q8 + (xcd < r8 ? xcd : r8) + slot;
    const unsigned z = fdiv(logical, g.dper_z), within = logical - z * (unsigned)g.per_z;
    const unsigned stile = within >> 5, in = within & 31;
    const unsigned srow = fdiv(stile, g.dnsc), scol = stile - srow * (unsigned)g.nsc;
    const int rb = (int)(srow * 8 + (in & 7)), cb = (int)(scol * 4 + (in >> 3));
    if (PADDED && (rb >= g.nrb || cb >= g.ncb)) return;     // padding slot of a ragged super-tile (whole workgroup)
    const unsigned zi1 = fdiv(z, g.dz0), zi0 = z - zi1 * (unsigned)g.z0;

    // Load j of a wave into a panel fills the 1 KB at 1024 (8 j + wave): 16-byte slot 64 (8 j + wave) + lane.
    unsigned offA[2], offB[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int slot16 = 64 * (8 * j + wave) + lane;
        offA[j] = 2 * wide_source<A_KC>(slot16, g.row.ld);
        offB[j] = 2 * wide_source<B_KC>(slot16, g.col.ld);
    }
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) uint16_t *)lds;
    const unsigned land = __builtin_amdgcn_readfirstlane(lds0 + wave * 1024);

    // Where the block's panels lie: lane i decodes panel i of the side (one pass of vector arithmetic for all
    // of them; a scalar odometer over ten panels would hold the loads back by hundreds of dependent
    // instructions) and the results are broadcast into wave-uniform registers.
    auto uniform64 = [](int64_t v, int src) __attribute__((always_inline)) {
        const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(uint32_t)v, src);
        const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)v >> 32), src);
        return (int64_t)(((uint64_t)hi << 32) | lo);
    };
    // every load of the block, in the order of need: A0, A1, B0, then B1 .. B7
    int64_t offA_p[WR], offC_r[WR], offB_s[WC], offC_s[WC];
    const Loc mine_r = locate1(g.row, rb * WR + (lane & (WR - 1)), g.R);
#pragma unroll
    for (int p = 0; p < WR; ++p) { offA_p[p] = uniform64(mine_r.off, p);  offC_r[p] = uniform64(mine_r.offC, p); }
    const uint16_t *Az = g.A + (int64_t)zi0 * g.zA[0] + (int64_t)zi1 * g.zA[1];
#pragma unroll
    for (int p = 0; p < WR; ++p)
#pragma unroll
        for (int j = 0; j < 2; ++j) dma16(land + p * (WPANEL * 2) + j * 8192, Az + offA_p[p], offA[j]);
    const Loc mine_c = locate1(g.col, cb * WC + (lane & (WC - 1)), g.Cn);
#pragma unroll
    for (int s = 0; s < WC; ++s) { offB_s[s] = uniform64(mine_c.off, s);  offC_s[s] = uniform64(mine_c.offC, s); }
    const uint16_t *Bz = g.B + (int64_t)zi0 * g.zB[0] + (int64_t)zi1 * g.zB[1];
    auto request_b = [&](int s) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < 2; ++j) dma16(land + (WR + s) * (WPANEL * 2) + j * 8192, Bz + offB_s[s], offB[j]);
    };
    static_assert(WAHEAD == 4, "the start-up below requests column panels 0 .. 3");
    request_b(0);

    // wave w: row panel w % 2, columns 16 (w / 2) .. +15 of every column panel
    const int pi = wave & 1, q = wave >> 1;
    const float alpha = g.alpha;
    uint16_t *Crow = g.C + (int64_t)zi0 * g.zC[0] + (int64_t)zi1 * g.zC[1] + (pi ? offC_r[1] : offC_r[0]) + (int64_t)(q * 16) * g.ldc;
    uint16_t *st = ldsA + wave * (2 * WSTAGE);

    // Start-up: the A fragments are 16 KB of LDS reads per wave (half a microsecond for the eight of them), so
    // they start as soon as the wave's row panel is there, while the next panels are still on their way: row
    // panel 0, row panel 1 and column panel 0 each get their own wait (always two younger panels) and barrier.
    // These barriers only publish what the loads wrote; they must not wait for the fragment reads in flight,
    // hence no fence (the empty asm statements keep the compiler from moving LDS accesses across).
    auto publish = [&]() __attribute__((always_inline)) {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    bf16x8 fa[4][4], fb[4];
    auto read_a = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int rt = 0; rt < 4; ++rt) fa[rt][ks] = wide_fragment<A_KC>(ldsA + pi * WPANEL, rt * 16, ks, lane);
    };
    dma_wait<4>();               // behind A0: A1, B0
    publish();
    if (pi == 0) read_a();
    request_b(1);
    dma_wait<4>();               // behind A1: B0, B1
    publish();
    if (pi == 1) read_a();
    request_b(2);
    dma_wait<4>();               // behind B0: B1, B2
    publish();
    request_b(3);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) fb[ks] = wide_fragment<B_KC>(ldsB, q * 16, ks, lane);

    auto read_b = [&](bf16x8 (&fb)[4], int s) __attribute__((always_inline)) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) fb[ks] = wide_fragment<B_KC>(ldsB + s * WPANEL, q * 16, ks, lane);
    };
    // result register r of lane l: row 16 rt + 4 (l / 16) + r, column l % 16 of the wave's 64 x 16 piece
    auto clear = [&](f32x4 (&acc)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int rt = 0; rt < 4; ++rt) acc[rt] = f32x4{0.f, 0.f, 0.f, 0.f};
    };
    auto half_product = [&](f32x4 (&acc)[4], const bf16x8 (&fb)[4], int h) __attribute__((always_inline)) {
#pragma unroll
        for (int ks = 2 * h; ks < 2 * h + 2; ++ks)
#pragma unroll
            for (int rt = 0; rt < 4; ++rt) acc[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[rt][ks], fb[ks], acc[rt], 0, 0, 0);
    };
    // Staging area: [16 columns][64 rows], the 8-byte unit u of column j at position u ^ j, so that the 8-byte
    // writes of a half wave (16 columns x 2 units) and the 16-byte reads (2 columns x 8 pairs) cover all banks.
    auto stage = [&](const f32x4 (&acc)[4], int s) __attribute__((always_inline)) {
        const int j = lane & 15;
        uint16_t *area = st + (s & 1) * WSTAGE + j * TM;
#pragma unroll
        for (int rt = 0; rt < 4; ++rt) {
            u16x4 pk;
#pragma unroll
            for (int e = 0; e < 4; ++e) pk[e] = sb_f32_to_bf16(alpha * acc[rt][e]);
            *(u16x4 *)(area + (((4 * rt + (lane >> 4)) ^ j) << 2)) = pk;
        }
    };
    auto wave_fence = [&]() __attribute__((always_inline)) {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };
    // the staged product s as two 16-byte vectors per lane: whole 128-byte lines of C, 8 lanes to a column
    auto read_staged = [&](u32x4 (&o)[2], int s) __attribute__((always_inline)) {
        const uint16_t *area = st + (s & 1) * WSTAGE;
        const int pr = lane & 7;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int jj = 8 * t + (lane >> 3);
            const u32x4 v = *(const u32x4 *)(area + jj * TM + ((pr ^ (jj >> 1)) << 3));
            o[t] = (jj & 1) ? u32x4{v[2], v[3], v[0], v[1]} : v;          // an odd column holds its unit pairs swapped
        }
    };
    // exactly two store instructions per product and wave (the waits count them)
    auto write_out = [&](const u32x4 (&o)[2], int64_t offC) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
            SB_PANEL_STORE((u32x4u *)(Crow + offC + (int64_t)(8 * t + (lane >> 3)) * g.ldc + 8 * (lane & 7)), o[t]);
    };

    f32x4 acc0[4], acc1[4];
    clear(acc0);
    half_product(acc0, fb, 0);
    half_product(acc0, fb, 1);
    __syncthreads();             // every wave holds its A fragments: the staging areas may overwrite the A panels
    // One step: product s, finished in `done`, is rounded, staged and stored; then the next column panel is
    // waited for (wide_pending: vector-memory operations this wave has issued after that panel's loads), the
    // barrier publishes it, and product s+1 is multiplied.  The stores of a product thus never wait for a
    // panel, and the panel WAHEAD steps ahead is requested behind them (the memory pipeline of a compute unit
    // accepts a 1 KB load every ~25 clocks: a wave that issued all its loads up front would reach its first
    // wait 1.5 us into the kernel).
    auto step = [&](const f32x4 (&done)[4], f32x4 (&next)[4], auto s_c, int64_t offC) __attribute__((always_inline)) {
        constexpr int S = decltype(s_c)::value;
        stage(done, S);
        wave_fence();
        u32x4 o[2];
        read_staged(o, S);
        write_out(o, offC);
        wave_fence();
        if (S + 1 < WC) {
            if (S + WAHEAD < WC) request_b(S + WAHEAD);
            dma_wait<wide_pending(S)>();
            __syncthreads();
            read_b(fb, S + 1);
            clear(next);
            half_product(next, fb, 0);
            half_product(next, fb, 1);
        }
    };
    step(acc0, acc1, std::integral_constant<int, 0>(), offC_s[0]);
    step(acc1, acc0, std::integral_constant<int, 1>(), offC_s[1]);
    step(acc0, acc1, std::integral_constant<int, 2>(), offC_s[2]);
    step(acc1, acc0, std::integral_constant<int, 3>(), offC_s[3]);
    step(acc0, acc1, std::integral_constant<int, 4>(), offC_s[4]);
    step(acc1, acc0, std::integral_constant<int, 5>(), offC_s[5]);
    step(acc0, acc1, std::integral_constant<int, 6>(), offC_s[6]);
    step(acc1, acc0, std::integral_constant<int, 7>(), offC_s[7]);
}

// ---------------------------------------------------------------------------------------------
// host side: an sb_gemm2 problem as a panel grid

FastDiv make_fastdiv(uint32_t d)            // 1 <= d < 2^31
{
    uint32_t l = 0;
    while (l < 32 && ((uint64_t)1 << l) < d) ++l;
    const uint64_t m = (((uint64_t)1 << 32) * (((uint64_t)1 << l) - d)) / d + 1;
    return FastDiv{(uint32_t)m, l};
}

struct Grid {
    PanelArgs p;
    bool ok;
    bool a_kc, b_kc, ragged;
    bool wide;               // blocks of 2 x 8 panels for the wide-block kernel (else 4 x 4)
    int64_t blocks;          // launched workgroups (padding slots included)
    int64_t real_blocks;     // blocks that hold at least one panel pair
    double utilisation;      // panel pairs / (16 * real blocks)
};

// The wide-block kernel takes the problem if nothing needs a guard or a fix-up: k == 128, beta == 0, whole panels
// in whole blocks, 16-byte aligned addresses everywhere, lane offsets inside a panel that fit 32 bits.
bool wide_applies(const SbArgs &a, const PanelArgs &p, bool a_kc, bool b_kc)
{
    if (a.k != KMAX || a.beta != 0.0) return false;
    const Side &r = p.row, &c = p.col;
    if (r.full != TM || r.last != TM || c.full != TM || c.last != TM) return false;
    if (p.R % WR != 0 || p.Cn % WC != 0) return false;
    if (r.ld >= (1u << 24) || c.ld >= (1u << 24)) return false;
    auto al = [](int64_t v) { return v % 8 == 0; };
    if (((uintptr_t)p.A | (uintptr_t)p.B | (uintptr_t)p.C) % 16 != 0) return false;
    if (!al(r.ld) || !al(c.ld) || !al(a.ldc)) return false;
    if (!al(r.sf) || !al(r.s1) || !al(r.s2) || !al(c.sf) || !al(c.s1) || !al(c.s2)) return false;
    if (!al(r.cf) || !al(r.c1) || !al(r.c2) || !al(c.cf) || !al(c.c1) || !al(c.c2)) return false;
    for (int q = 0; q < 2; ++q)
        if (!al(p.zA[q]) || !al(p.zB[q]) || !al(p.zC[q])) return false;
    return true;
}

Grid make_grid(const SbArgs &a)
{
    Grid gr;
    gr.ok = false;
    if (a.k < 1 || a.k > KMAX || a.m < 1 || a.n < 1 || a.nx > 0) return gr;
    const bool a_kc = (a.csA == 1), b_kc = (a.rsB == 1);
    if (!a_kc && a.rsA != 1) return gr;
    if (!b_kc && a.csB != 1) return gr;
    PanelArgs &p = gr.p;
    p.A = (const uint16_t *)a.A;  p.B = (const uint16_t *)a.B;  p.C = (uint16_t *)a.C;
    Side &r = p.row, &c = p.col;
    auto flat = [](Side &s, int64_t extent, int64_t op_stride, int64_t c_stride, int64_t ld) {
        s.nf = (int32_t)((extent + 63) / 64);
        s.full = extent < 64 ? (int32_t)extent : 64;
        s.last = (int32_t)(extent - 64 * (int64_t)(s.nf - 1));
        s.sf = 64 * op_stride;  s.cf = 64 * c_stride;
        s.n1 = s.n2 = 1;  s.s1 = s.s2 = s.c1 = s.c2 = 0;
        s.ld = (uint32_t)ld;
    };
    const int64_t ldA = a_kc ? a.rsA : a.csA, ldB = b_kc ? a.csB : a.rsB;
    if (ldA < 0 || ldB < 0 || ldA >= ((int64_t)1 << 31) || ldB >= ((int64_t)1 << 31)) return gr;
    if (a.m > ((int64_t)1 << 36) || a.n > ((int64_t)1 << 36)) return gr;
    flat(r, a.m, a.rsA, 1, ldA);
    flat(c, a.n, a.csB, a.ldc, ldB);
    p.z0 = p.z1 = 1;
    for (int q = 0; q < 2; ++q) p.zA[q] = p.zB[q] = p.zC[q] = 0;
    int nz = 0;
    const int64_t cnt[2] = {a.batch0, a.batch1};
    for (int q = 0; q < 2; ++q) {
        if (cnt[q] <= 1) continue;
        if (cnt[q] >= ((int64_t)1 << 31)) return gr;
        const bool movesA = a.bsA[q] != 0, movesB = a.bsB[q] != 0;
        Side *s = (movesA && !movesB) ? &r : ((movesB && !movesA) ? &c : nullptr);
        if (s) {               // this level moves one operand only: it extends that operand's side
            const int64_t so = movesA ? a.bsA[q] : a.bsB[q];
            if (s->n1 == 1) { s->n1 = (int32_t)cnt[q]; s->s1 = so; s->c1 = a.bsC[q]; }
            else            { s->n2 = (int32_t)cnt[q]; s->s2 = so; s->c2 = a.bsC[q]; }
        } else {               // both operands (or neither) move: independent grids
            (nz == 0 ? p.z0 : p.z1) = (int32_t)cnt[q];
            p.zA[nz] = a.bsA[q];  p.zB[nz] = a.bsB[q];  p.zC[nz] = a.bsC[q];
            ++nz;
        }
    }
    const int64_t R = (int64_t)r.nf * r.n1 * r.n2, Cn = (int64_t)c.nf * c.n1 * c.n2;
    if (R >= ((int64_t)1 << 30) || Cn >= ((int64_t)1 << 30)) return gr;
    p.R = (int32_t)R;  p.Cn = (int32_t)Cn;
    p.ldc = a.ldc;
    gr.wide = wide_applies(a, p, a_kc, b_kc);
    // blocks of 4 x 4 panels in super-tiles of 4 x 8 blocks, or blocks of 2 x 8 panels in super-tiles of 8 x 4
    const int br = gr.wide ? WR : BR, bc = gr.wide ? WC : BC;
    p.nrb = (int32_t)((R + br - 1) / br);  p.ncb = (int32_t)((Cn + bc - 1) / bc);
    const int64_t nsr = gr.wide ? (p.nrb + 7) / 8 : (p.nrb + 3) / 4, nsc = gr.wide ? (p.ncb + 3) / 4 : (p.ncb + 7) / 8;
    p.nsc = (int32_t)nsc;
    const int64_t per_z = nsr * nsc * 32, Z = (int64_t)p.z0 * p.z1;
    if (per_z >= ((int64_t)1 << 31) || per_z * Z > sb_max_grid_x(NT)) return gr;
    p.per_z = (int32_t)per_z;
    r.dnf = make_fastdiv((uint32_t)r.nf);  r.dn1 = make_fastdiv((uint32_t)r.n1);
    c.dnf = make_fastdiv((uint32_t)c.nf);  c.dn1 = make_fastdiv((uint32_t)c.n1);
    p.dper_z = make_fastdiv((uint32_t)per_z);  p.dnsc = make_fastdiv((uint32_t)nsc);  p.dz0 = make_fastdiv((uint32_t)p.z0);
    p.k = (int32_t)a.k;
    p.alpha = (float)a.alpha;  p.beta = (float)a.beta;
    gr.a_kc = a_kc;  gr.b_kc = b_kc;
    // whole 16-byte vectors along the contiguous direction of both operands and of C
    gr.ragged = (a_kc ? a.k % 8 != 0 : (r.full % 8 || r.last % 8)) || (b_kc ? a.k % 8 != 0 : (c.full % 8 || c.last % 8)) ||
                r.full % 8 || r.last % 8;
    gr.blocks = per_z * Z;
    gr.real_blocks = (int64_t)p.nrb * p.ncb * Z;
    gr.utilisation = (double)(R * Cn) / (double)(16 * (int64_t)p.nrb * p.ncb);         // 16 panel pairs per block of either shape
    gr.ok = true;
    return gr;
}

template <bool A_KC, bool B_KC>
hipError_t launch_grid(const Grid &gr, hipStream_t stream)
{
    const size_t lds_bytes = (size_t)(gr.wide ? WLDS_ELEMS : LDS_ELEMS) * sizeof(uint16_t);
    const dim3 grid((unsigned)gr.blocks), block(NT);
#define SB_PANELGRID(KS_, RG_) SB_PANELGRID_KERNEL((sbgemm_panelgrid_bf16_kernel<A_KC, B_KC, KS_, RG_>))
#define SB_PANELGRID_KERNEL(KERNEL_)                                                                                    \
    do {                                                                                                                \
        auto kern = KERNEL_;                                                                                            \
        static std::atomic<bool> configured[SB_MAX_DEVICES] = {};                                                       \
        const int dev = sb_current_device();                                                                            \
        if (!configured[dev]) {                                                                                         \
            hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes); \
            if (e != hipSuccess) return e;                                                                              \
            configured[dev] = true;                                                                                     \
        }                                                                                                               \
        hipLaunchKernelGGL(kern, grid, block, lds_bytes, stream, gr.p);                                                 \
    } while (0)
    const bool short_k = gr.p.k <= 64;
    if (gr.wide && gr.blocks == gr.real_blocks) SB_PANELGRID_KERNEL((sbgemm_panelgrid_wide_bf16_kernel<A_KC, B_KC, false>));
    else if (gr.wide) SB_PANELGRID_KERNEL((sbgemm_panelgrid_wide_bf16_kernel<A_KC, B_KC, true>));
    else if (gr.ragged) { if (short_k) SB_PANELGRID(4, true);  else SB_PANELGRID(8, true); }
    else           { if (short_k) SB_PANELGRID(4, false); else SB_PANELGRID(8, false); }
#undef SB_PANELGRID
#undef SB_PANELGRID_KERNEL
    return hipGetLastError();
}

}  // namespace

// Can run: bf16 (the caller checks the type), 1 <= k <= 128, each operand contiguous along k or along
// its rows (columns), grid within launch limits.
bool sb_panel_bf16_supports(const SbArgs &a)
{
    return make_grid(a).ok;
}

// Should run: at least 4 panels on both sides, blocks mostly full, and enough blocks to occupy half the
// chip (a block keeps one compute unit busy).  Smaller problems are better off on 64 x 64 tiles.
bool sb_panel_bf16_preferred(const SbArgs &a)
{
    const Grid gr = make_grid(a);
    return gr.ok && gr.p.R >= 4 && gr.p.Cn >= 4 && gr.utilisation >= 0.55 && gr.real_blocks >= 128;
}

hipError_t sb_launch_panel_bf16(const SbArgs &a, hipStream_t stream)
{
    const Grid gr = make_grid(a);
    if (!gr.ok) return hipErrorInvalidValue;
    sb_note_member(gr.wide ? SB_MEMBER_PANEL_WIDE : SB_MEMBER_PANEL_4X4);
    if (gr.a_kc && gr.b_kc)  return launch_grid<true, true>(gr, stream);
    if (gr.a_kc && !gr.b_kc) return launch_grid<true, false>(gr, stream);
    if (!gr.a_kc && gr.b_kc) return launch_grid<false, true>(gr, stream);
    return launch_grid<false, false>(gr, stream);
}
