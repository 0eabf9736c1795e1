// Whole-K panel kernel for nests of small bf16 GEMMs (m, n <= 64, k <= 128) whose two batch
// levels each move one operand: the batch loops take part in the tiling (section III-D argues a
// strided batch interface allows exactly this; section III-F, Listing 2 is the nested case).
#include "sb_device.h"
#include "sb_internal.h"

#include <atomic>


namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));

constexpr int TM = 64, TN = 64, KMAX = 128;
constexpr int LD_KC = KMAX + 8;          // [row][k] layout, rows padded by 16 bytes

// Two-level ("outer product") batch blocking: op(A) depends only on batch level 0 and op(B) only
// on level 1, as in C_mn[p][q] = A_mk[p] B_nk[q] (section III-F).  The (p,q) batches then form a
// grid in which every A_p meets every B_q, and a workgroup that takes a 2 x 2 block of that grid
// needs only 2 + 2 panels for 4 small GEMMs: the nested batch becomes a blocked computation with
// operand reuse, although no operand is ever flattened or copied.  Four waves, one GEMM of up to
// 64 x 64 x 128 each; 68 KB of LDS, so two workgroups share a compute unit and one block's
// stores drain to HBM while the next block's panels are being fetched.
// Every panel is kept [row][k] in LDS, whatever the operand's orientation in memory, so that an
// MFMA operand is always ONE 16-byte LDS read (a [k][row] panel needs eight 2-byte reads per
// operand).  An operand with m (or n) contiguous is transposed on the
// way in: a lane loads an 8 x 8 block (8 vectors of 8 rows, one per k), transposes it in registers
// and writes 8 vectors of 8 k.  Those rows are 8 apart for neighbouring lanes, which a plain
// layout would put on the same banks; the 16-byte chunk index of such a panel is therefore XORed
// with (row / 8) % 8, on the write and on the read side.
constexpr int GP2 = 2, GQ2 = 2, OT2 = 256;
constexpr int PANEL2 = TM * LD_KC;                            // elements; [row][k], rows padded by 16 bytes
constexpr int SPITCH2 = 68;                                   // staged column: 64 rows + 8 bytes
constexpr int OUTER2_LDS = (GP2 + GQ2) * PANEL2;              // the staging area (4 x 64 x 68 elements) fits inside

// The two panels of one operand (X_{b0}, X_{b0+1}) on their way from memory to LDS, spread over all
// 256 lanes: load() only issues the global loads (so that the panels of a later block can already be
// in flight), store() writes them to LDS in [row][k] form.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <bool KC>
struct TwoPanels {
    u32x4 v[8];

    __device__ __forceinline__ void load(const uint16_t *X, int64_t bs, int64_t b0, int64_t blim, int64_t ld, int rows, int kk)
    {
        const int tid = (int)threadIdx.x;
        if (KC) {                       // k contiguous in memory: 2 x 1024 vectors, straight copy
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int panel = i / 4, f = tid + OT2 * (i % 4);
                const int row = f / (KMAX / 8), k = (f % (KMAX / 8)) * 8;
                int64_t b = b0 + panel;
                if (b >= blim) b = blim - 1;          // past the end: any valid panel, its results are never stored
                const bool inside = row < rows && k < kk;
                v[i] = *(const u32x4 *)(X + b * bs + (inside ? (int64_t)row * ld + k : 0));
            }
        } else {                        // rows contiguous in memory: one 8 x 8 block per lane (8 vectors of 8 rows)
            const int panel = tid / 128, blk = tid % 128;
            const int rg = blk % 8, kg = blk / 8;                  // rows 8 rg .. +7, k 8 kg .. +7
            int64_t b = b0 + panel;
            if (b >= blim) b = blim - 1;
            const uint16_t *src = X + b * bs;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int k = kg * 8 + i;
                const bool inside = rg * 8 < rows && k < kk;
                v[i] = *(const u32x4 *)(src + (inside ? (int64_t)k * ld + rg * 8 : 0));
            }
        }
    }

    // vectors outside the matrix become zeros here (not after the load, which would wait for it)
    __device__ __forceinline__ void store(uint16_t *lds, int rows, int kk) const
    {
        const int tid = (int)threadIdx.x;
        const u32x4 z = {0, 0, 0, 0};
        if (KC) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int panel = i / 4, f = tid + OT2 * (i % 4);
                const int row = f / (KMAX / 8), k = (f % (KMAX / 8)) * 8;
                *(u32x4 *)(lds + panel * PANEL2 + row * LD_KC + k) = (row < rows && k < kk) ? v[i] : z;
            }
        } else {                        // transposed in registers: row 8 rg + j gets its 8 k as 4 words
            const int panel = tid / 128, blk = tid % 128;
            const int rg = blk % 8, kg = blk / 8;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                u32x4 w;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const bool in_lo = rg * 8 < rows && kg * 8 + 2 * c < kk, in_hi = rg * 8 < rows && kg * 8 + 2 * c + 1 < kk;
                    const unsigned lo = in_lo ? v[2 * c][j / 2] : 0u, hi = in_hi ? v[2 * c + 1][j / 2] : 0u;
                    w[c] = (j % 2 == 0) ? ((lo & 0xffffu) | (hi << 16)) : ((lo >> 16) | (hi & 0xffff0000u));
                }
                *(u32x4 *)(lds + panel * PANEL2 + (rg * 8 + j) * LD_KC + ((kg ^ rg) * 8)) = w;
            }
        }
    }
};

// MFMA operand of the 32 rows starting at row0 for k-step ks; SWZ: the panel was written with the chunk swizzle
template <bool SWZ>
__device__ __forceinline__ bf16x8 panel2_fragment(const uint16_t *lds, int row0, int ks, int lane)
{
    const int row = row0 + (lane & 31);
    int chunk = ks * 2 + (lane >> 5);
    if (SWZ) chunk ^= (row >> 3) & 7;
    return __builtin_bit_cast(bf16x8, *(const u16x8 *)(lds + row * LD_KC + chunk * 8));
}

// A workgroup takes TWO neighbouring 2 x 2 blocks (same A panels, the next two B panels).  The loads of
// the second block's B panels are issued together with the first block's, so they are in flight
// while the first block is multiplied and stored, and the first block's stores drain while the
// second is multiplied: with one block per workgroup the grid ran as two rounds of workgroups whose
// fetch, multiply and store phases (2.4 + 1.0 + 2.0 us, each a chain of latencies) simply added up.
template <bool A_KC, bool B_KC, int KS>
__global__ __launch_bounds__(OT2) void sbgemm_outer2_bf16_kernel(SbArgs g, int groups_p, int vec_store)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];      // [A0 A1 | B0 B1]; the B half doubles as staging area
    const int gp = (int)(blockIdx.x % groups_p), gq2 = (int)(blockIdx.x / groups_p);
    const int64_t p0 = (int64_t)gp * GP2, q0 = (int64_t)gq2 * (2 * GQ2);
    const int m = (int)g.m, n = (int)g.n, kk = (int)g.k;
    const int64_t ldA = A_KC ? g.rsA : g.csA, ldB = B_KC ? g.csB : g.rsB;
    uint16_t *ldsB = lds + GP2 * PANEL2;

    TwoPanels<A_KC> pa;
    TwoPanels<B_KC> pb, pb2;
    pa.load((const uint16_t *)g.A, g.bsA[0], p0, g.batch0, ldA, m, kk);
    pb.load((const uint16_t *)g.B, g.bsB[1], q0, g.batch1, ldB, n, kk);
    pb2.load((const uint16_t *)g.B, g.bsB[1], q0 + GQ2, g.batch1, ldB, n, kk);      // clamped when there is no second block
    pa.store(lds, m, kk);
    pb.store(ldsB, n, kk);
    __syncthreads();

    // wave w: the whole 64 x 64 GEMM A_{p0 + w/2} B_{q + w%2}
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int pi = wave >> 1, qi = wave & 1;
    const uint16_t *la = lds + pi * PANEL2, *lb = ldsB + qi * PANEL2;
    const float alpha = (float)g.alpha, beta = (float)g.beta;
    const int64_t p = p0 + pi;
    uint16_t *st = ldsB + wave * (TN * SPITCH2);
    typedef unsigned short u16x4 __attribute__((ext_vector_type(4)));

    // multiply, park the results as bf16 in the B half (free once every wave has its products),
    // write whole 128-byte lines of C
    auto block = [&](int64_t q) {
        f32x16 acc[2][2];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[a][c][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            bf16x8 fa[2], fb[2];
#pragma unroll
            for (int a = 0; a < 2; ++a) fa[a] = panel2_fragment<!A_KC>(la, a * 32, ks, lane);
#pragma unroll
            for (int c = 0; c < 2; ++c) fb[c] = panel2_fragment<!B_KC>(lb, c * 32, ks, lane);
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int c = 0; c < 2; ++c)
                    // result register r of lane l: row 8 (r/4) + 4 (l/32) + r%4, column l%32 of the 32 x 32 block
                    acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[c], acc[a][c], 0, 0, 0);
        }
        __syncthreads();             // every wave is done with the B panels
        const bool live = p < g.batch0 && q < g.batch1;
        uint16_t *Cq = (uint16_t *)g.C + (live ? p * g.bsC[0] + q * g.bsC[1] : 0);
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const int j = c * 32 + (lane & 31);
#pragma unroll
                for (int gq4 = 0; gq4 < 4; ++gq4) {
                    const int i0 = a * 32 + 8 * gq4 + 4 * (lane >> 5);
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = alpha * acc[a][c][4 * gq4 + e];
                    if (beta != 0.f && live && j < n) {
                        const uint16_t *old = Cq + (int64_t)j * g.ldc + i0;
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (i0 + e < m) v[e] += beta * sb_bf16_to_f32(old[e]);
                    }
                    u16x4 pk;
#pragma unroll
                    for (int e = 0; e < 4; ++e) pk[e] = sb_f32_to_bf16(v[e]);
                    *(u16x4 *)(st + j * SPITCH2 + i0) = pk;
                }
            }
        __syncthreads();
        if (live) {
            if (vec_store) {             // m is a multiple of 8 and every column of C starts 16-byte aligned
                const int seg = 8 * (lane & 7);
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const int j = 8 * t + (lane >> 3);
                    const u16x4 lo = *(const u16x4 *)(st + j * SPITCH2 + seg);
                    const u16x4 hi = *(const u16x4 *)(st + j * SPITCH2 + seg + 4);
                    if (seg < m && j < n) {
                        u16x8 o = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                        *(u16x8 *)(Cq + (int64_t)j * g.ldc + seg) = o;
                    }
                }
            } else {
#pragma unroll 4
                for (int j = 0; j < TN; ++j) {
                    const uint16_t v = st[j * SPITCH2 + lane];
                    if (lane < m && j < n) Cq[(int64_t)j * g.ldc + lane] = v;
                }
            }
        }
    };

    block(q0 + qi);
    if (q0 + GQ2 < g.batch1) {           // workgroup-uniform: the second block exists
        __syncthreads();                 // the staged results of the first block have been read
        pb2.store(ldsB, n, kk);
        __syncthreads();
        block(q0 + GQ2 + qi);
    }
}

}  // namespace

static bool outer_applies(const SbArgs &a);

bool sb_panel_bf16_supports(const SbArgs &a)
{
    if (a.batch0 * a.batch1 >= ((int64_t)1 << 31)) return false;
    if (a.m > TM || a.n > TN || a.k > KMAX || a.k <= 0) return false;
    const bool a_kc = (a.csA == 1), b_kc = (a.rsB == 1);
    if (!a_kc && a.rsA != 1) return false;
    if (!b_kc && a.csB != 1) return false;
    auto al = [](int64_t v) { return v % 8 == 0; };
    // 16-byte vector loads: aligned bases and strides, whole vectors along the contiguous dimension
    if ((uintptr_t)a.A % 16 || (uintptr_t)a.B % 16) return false;
    if (!al(a_kc ? a.rsA : a.csA) || !al(b_kc ? a.csB : a.rsB)) return false;
    if (!al(a.bsA[0]) || !al(a.bsA[1]) || !al(a.bsB[0]) || !al(a.bsB[1])) return false;
    if (a_kc ? !al(a.k) : !al(a.m)) return false;
    if (b_kc ? !al(a.k) : !al(a.n)) return false;
    return outer_applies(a);
}

template <bool A_KC, bool B_KC>
static hipError_t launch_outer(const SbArgs &a, hipStream_t stream)
{
    auto al8 = [](int64_t v) { return v % 8 == 0; };
    const int vec_store = (uintptr_t)a.C % 16 == 0 && al8(a.ldc) && al8(a.bsC[0]) && al8(a.bsC[1]) && al8(a.m);
    const int ks = (int)((a.k + 15) / 16);
    const int64_t groups_p = (a.batch0 + GP2 - 1) / GP2, groups_q = (a.batch1 + 2 * GQ2 - 1) / (2 * GQ2);     // two blocks along q per workgroup
    const size_t lds_bytes = (size_t)OUTER2_LDS * sizeof(uint16_t);
    dim3 grid((unsigned)(groups_p * groups_q)), block(OT2);
#define SB_OUTER(KS_)                                                                                                  \
    do {                                                                                                                \
        auto kern = sbgemm_outer2_bf16_kernel<A_KC, B_KC, KS_>;                                                         \
        static std::atomic<bool> configured[SB_MAX_DEVICES] = {};                                                                    \
        const int dev = sb_current_device();                                                                            \
        if (!configured[dev]) {                                                                                         \
            hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes); \
            if (e != hipSuccess) return e;                                                                              \
            configured[dev] = true;                                                                                     \
        }                                                                                                               \
        hipLaunchKernelGGL(kern, grid, block, lds_bytes, stream, a, (int)groups_p, vec_store);                          \
    } while (0)
    if (ks <= 2)      SB_OUTER(2);
    else if (ks <= 4) SB_OUTER(4);
    else              SB_OUTER(8);
#undef SB_OUTER
    return hipGetLastError();
}

// A varies only with batch level 0 and B only with level 1 (both really vary), enough of both
static bool outer_applies(const SbArgs &a)
{
    return a.batch0 >= 4 && a.batch1 >= 4 && a.bsA[1] == 0 && a.bsB[0] == 0 && a.bsA[0] != 0 && a.bsB[1] != 0 &&
           a.batch0 * a.batch1 / (GP2 * GQ2) < ((int64_t)1 << 30);
}

hipError_t sb_launch_panel_bf16(const SbArgs &a, hipStream_t stream)
{
    const bool ak = a.csA == 1, bk = a.rsB == 1;
    if (ak && bk)  return launch_outer<true, true>(a, stream);
    if (ak && !bk) return launch_outer<true, false>(a, stream);
    if (!ak && bk) return launch_outer<false, true>(a, stream);
    return launch_outer<false, false>(a, stream);
}
