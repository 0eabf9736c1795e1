// Whole-K panel kernel for nests of small bf16 GEMMs (m, n <= 64, k <= 128) whose two batch
// levels each move one operand: the batch loops take part in the tiling (section III-D argues a
// strided batch interface allows exactly this; section III-F, Listing 2 is the nested case).
#include "sb_device.h"
#include "sb_internal.h"


namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));

constexpr int TM = 64, TN = 64, KMAX = 128;
constexpr int LD_KC = KMAX + 8;          // [row][k] layout, rows padded by 16 bytes
constexpr int LD_MC = TM + 8;            // [k][row] layout
constexpr int PANEL = (TM * LD_KC > KMAX * LD_MC) ? TM * LD_KC : KMAX * LD_MC;   // elements

// MFMA operand of the 32 rows starting at row0 for k-step ks: lane l holds X[row0 + l%32][16 ks + 8 (l/32) .. +7]
template <bool KC>
__device__ __forceinline__ bf16x8 panel_fragment(const uint16_t *lds, int row0, int ks, int lane)
{
    const int row = row0 + (lane & 31);
    const int k = ks * 16 + (lane >> 5) * 8;
    u16x8 v;
    if (KC) {
        v = *(const u16x8 *)(lds + row * LD_KC + k);
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = lds[(k + e) * LD_MC + row];
    }
    return __builtin_bit_cast(bf16x8, v);
}

// Two-level ("outer product") batch blocking: op(A) depends only on batch level 0 and op(B) only
// on level 1, as in C_mn[p][q] = A_mk[p] B_nk[q] (section III-F).  The (p,q) batches then form a
// grid in which every A_p meets every B_q, and a workgroup that takes a GP x GQ block of that grid
// needs only GP + GQ panels for GP*GQ small GEMMs: the nested batch becomes a blocked computation
// with the operand reuse of a large GEMM, although no operand is ever flattened or copied.
// One workgroup of 16 waves: 4 + 4 whole-K panels in LDS (all eight fetched at once, which also
// puts enough bytes in flight to cover memory latency), 16 GEMMs of up to 64 x 64 x 128.
constexpr int GP = 4, GQ = 4, OT = 1024;
constexpr int ONVEC = (GP + GQ) * TM * KMAX / 8 / OT;     // 16-byte vectors per lane for all panels (8)

// Results leave through LDS: a wave parks its 32 x 64 x 2 block as bf16, column by column, and
// writes it out as 16-byte vectors along the rows of C (64 two-byte stores per lane become 8).
constexpr int SPITCH = 36;                        // elements per staged column: 32 rows + 8 bytes (bank spread)
constexpr int STAGE = 2 * TN * SPITCH;            // per wave: two GEMMs x 64 columns
constexpr int OUTER_LDS = ((GP + GQ) * PANEL > (OT / 64) * STAGE) ? (GP + GQ) * PANEL : (OT / 64) * STAGE;   // elements

template <bool A_KC, bool B_KC, int KS>
__global__ __launch_bounds__(OT) void sbgemm_outer_bf16_kernel(SbArgs g, int groups_p, int vec_store)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];      // [GP + GQ][PANEL], later [wave][STAGE]
    const int gp = (int)(blockIdx.x % groups_p), gq = (int)(blockIdx.x / groups_p);
    const int64_t p0 = (int64_t)gp * GP, q0 = (int64_t)gq * GQ;
    const int m = (int)g.m, n = (int)g.n, kk = (int)g.k;
    const int64_t ldA = A_KC ? g.rsA : g.csA, ldB = B_KC ? g.csB : g.rsB;

    // fill: panel j < GP is A_{p0+j}, panel GP + j is B_{q0+j}; indices past the end are clamped
    // (their results are never stored)
    {
        u16x8 v[ONVEC];
#pragma unroll
        for (int i = 0; i < ONVEC; ++i) {
            const int panel = i;                               // lane handles one vector slot of every panel
            const int f = (int)threadIdx.x;
            const bool is_a = panel < GP;
            const bool kc = is_a ? A_KC : B_KC;
            int row, k;
            if (kc) { row = f / (KMAX / 8); k = (f % (KMAX / 8)) * 8; }
            else    { k = f / (TM / 8); row = (f % (TM / 8)) * 8; }
            const int rows = is_a ? m : n;
            const bool inside = row < rows && k < kk;
            int64_t b = is_a ? p0 + panel : q0 + (panel - GP);
            const int64_t lim = is_a ? g.batch0 : g.batch1;
            if (b >= lim) b = lim - 1;
            const uint16_t *base = is_a ? (const uint16_t *)g.A + b * g.bsA[0] : (const uint16_t *)g.B + b * g.bsB[1];
            const int64_t ld = is_a ? ldA : ldB;
            const int64_t off = kc ? (int64_t)row * ld + k : (int64_t)k * ld + row;
            v[i] = *(const u16x8 *)(base + (inside ? off : 0));
        }
#pragma unroll
        for (int i = 0; i < ONVEC; ++i) {
            const int panel = i;
            const int f = (int)threadIdx.x;
            const bool is_a = panel < GP;
            const bool kc = is_a ? A_KC : B_KC;
            int row, k;
            if (kc) { row = f / (KMAX / 8); k = (f % (KMAX / 8)) * 8; }
            else    { k = f / (TM / 8); row = (f % (TM / 8)) * 8; }
            const int rows = is_a ? m : n;
            const u16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
            uint16_t *dst = lds + panel * PANEL + (kc ? row * LD_KC + k : k * LD_MC + row);
            *(u16x8 *)dst = (row < rows && k < kk) ? v[i] : z;
        }
    }
    __syncthreads();

    // wave w: A panel w/4, row block (w/2)%2, the two B panels 2*(w%2) and 2*(w%2)+1, both column blocks
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int pi = wave >> 2, rb = (wave >> 1) & 1, qh = wave & 1;
    const uint16_t *la = lds + pi * PANEL;
    f32x16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][c][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 fa = panel_fragment<A_KC>(la, rb * 32, ks, lane);
#pragma unroll
        for (int qq = 0; qq < 2; ++qq) {
            const uint16_t *lb = lds + (GP + 2 * qh + qq) * PANEL;
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                const bf16x8 fb = panel_fragment<B_KC>(lb, cb * 32, ks, lane);
                // result register r of lane l: row 8 (r/4) + 4 (l/32) + r%4, column l%32 of the 32 x 32 block
                acc[qq][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc[qq][cb], 0, 0, 0);
            }
        }
    }
    __syncthreads();                 // every wave is done with the panels: the space becomes the staging area

    const float alpha = (float)g.alpha, beta = (float)g.beta;
    const int64_t p = p0 + pi;
    const int row0 = rb * 32;
    uint16_t *st = lds + wave * STAGE;
    uint16_t *Cp = (uint16_t *)g.C + p * g.bsC[0] + row0;
#pragma unroll
    for (int qq = 0; qq < 2; ++qq) {
        const int64_t q = q0 + 2 * qh + qq;
        const bool live = p < g.batch0 && q < g.batch1;
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            const int j = cb * 32 + (lane & 31);
#pragma unroll
            for (int gq4 = 0; gq4 < 4; ++gq4) {
                const int i0 = 8 * gq4 + 4 * (lane >> 5);
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = alpha * acc[qq][cb][4 * gq4 + e];
                if (beta != 0.f && live && j < n) {
                    const uint16_t *old = Cp + q * g.bsC[1] + (int64_t)j * g.ldc + i0;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (row0 + i0 + e < m) v[e] += beta * sb_bf16_to_f32(old[e]);
                }
                typedef unsigned short u16x4 __attribute__((ext_vector_type(4)));
                u16x4 pk;
#pragma unroll
                for (int e = 0; e < 4; ++e) pk[e] = sb_f32_to_bf16(v[e]);
                *(u16x4 *)(st + (qq * TN + j) * SPITCH + i0) = pk;
            }
        }
    }
    __syncthreads();
#pragma unroll
    for (int qq = 0; qq < 2; ++qq) {
        const int64_t q = q0 + 2 * qh + qq;
        if (!(p < g.batch0 && q < g.batch1)) continue;
        uint16_t *Cq = Cp + q * g.bsC[1];
        const uint16_t *sq = st + qq * TN * SPITCH;
        if (vec_store) {             // m is a multiple of 8 and every column of C starts 16-byte aligned
            typedef unsigned short u16x4 __attribute__((ext_vector_type(4)));
            const int seg = 8 * (lane & 3);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int j = 16 * t + (lane >> 2);
                const u16x4 lo = *(const u16x4 *)(sq + j * SPITCH + seg);
                const u16x4 hi = *(const u16x4 *)(sq + j * SPITCH + seg + 4);
                if (row0 + seg < m && j < n) {
                    u16x8 o = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    *(u16x8 *)(Cq + (int64_t)j * g.ldc + seg) = o;
                }
            }
        } else {
            const int i = lane & 31;
#pragma unroll 4
            for (int jj = 0; jj < TN; jj += 2) {
                const int j = jj + (lane >> 5);
                const uint16_t v = sq[j * SPITCH + i];
                if (row0 + i < m && j < n) Cq[(int64_t)j * g.ldc + i] = v;
            }
        }
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
    const int64_t groups_p = (a.batch0 + GP - 1) / GP, groups_q = (a.batch1 + GQ - 1) / GQ;
    const size_t lds_bytes = (size_t)OUTER_LDS * sizeof(uint16_t);
    auto al8 = [](int64_t v) { return v % 8 == 0; };
    const int vec_store = (uintptr_t)a.C % 16 == 0 && al8(a.ldc) && al8(a.bsC[0]) && al8(a.bsC[1]) && al8(a.m);
    dim3 grid((unsigned)(groups_p * groups_q)), block(OT);
    const int ks = (int)((a.k + 15) / 16);
#define SB_OUTER(KS_)                                                                                                  \
    do {                                                                                                                \
        auto kern = sbgemm_outer_bf16_kernel<A_KC, B_KC, KS_>;                                                          \
        static bool configured = false;                                                                                 \
        if (!configured) {                                                                                              \
            hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes); \
            if (e != hipSuccess) return e;                                                                              \
            configured = true;                                                                                          \
        }                                                                                                               \
        hipLaunchKernelGGL(kern, grid, block, lds_bytes, stream, a, (int)groups_p, vec_store);                               \
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
           a.batch0 * a.batch1 / (GP * GQ) < ((int64_t)1 << 30);
}

hipError_t sb_launch_panel_bf16(const SbArgs &a, hipStream_t stream)
{
    const bool ak = a.csA == 1, bk = a.rsB == 1;
    if (ak && bk)  return launch_outer<true, true>(a, stream);
    if (ak && !bk) return launch_outer<true, false>(a, stream);
    if (!ak && bk) return launch_outer<false, true>(a, stream);
    return launch_outer<false, false>(a, stream);
}
