// C-ABI front end: argument validation, normalisation of the operations into strides, kernel
// selection and launch (section III-D, Listing 1; section III-F, Listing 2).
#include "sb_internal.h"

#include <algorithm>
#include <cstring>

namespace {

// diagnostics state is per host thread: a thread pins and reads the family of its own calls
thread_local int g_force_kernel = SB_KERNEL_AUTO;
thread_local int g_last_kernel = -1;
thread_local int g_last_member = 0;

bool valid_op(int op) { return op >= SB_OP_N && op <= SB_OP_EX_T; }
bool is_ex(int op) { return op == SB_OP_EX_N || op == SB_OP_EX_T; }

// Strides of op(X)(row, col) for a stored matrix described by (op, ld, stride0).
void op_strides(int op, int64_t ld, int64_t stride0, int64_t &rs, int64_t &cs, int64_t &bs0)
{
    switch (op) {
    case SB_OP_N:    rs = 1;       cs = ld;      bs0 = stride0; break;
    case SB_OP_T:    rs = ld;      cs = 1;       bs0 = stride0; break;
    case SB_OP_EX_N: rs = ld;      cs = stride0; bs0 = 1;       break;   // section III-E
    default:         rs = stride0; cs = ld;      bs0 = 1;       break;   // SB_OP_EX_T
    }
}

// The selector: which kernel family runs a problem (host arithmetic on sizes and strides only).
int choose(sb_dtype dt, const SbArgs &a, int forced)
{
    if (forced == SB_KERNEL_TINY && sb_tiny_supports(dt, a)) return SB_KERNEL_TINY;
    if (forced == SB_KERNEL_MFMA && sb_mfma_supports(dt, a)) return SB_KERNEL_MFMA;
    if (forced == SB_KERNEL_THIN && sb_thin_supports(dt, a)) return SB_KERNEL_THIN;
    if (forced == SB_KERNEL_PANEL && dt == SB_BF16 && sb_panel_bf16_supports(a)) return SB_KERNEL_PANEL;
    if (forced == SB_KERNEL_AUTO) {
        if (sb_thin_supports(dt, a) && sb_thin_preferred(dt, a)) return SB_KERNEL_THIN;
        if (sb_tiny_supports(dt, a) && sb_tiny_preferred(dt, a)) return SB_KERNEL_TINY;
        if (dt == SB_BF16 && sb_panel_bf16_preferred(a)) return SB_KERNEL_PANEL;
        if (sb_mfma_supports(dt, a) && sb_mfma_preferred(dt, a)) return SB_KERNEL_MFMA;
    }
    return SB_KERNEL_GENERIC;
}

// No two index tuples (i, j, p0, p1, ..) may address the same element of C.  Sufficient test: sorted by
// stride, each direction (rows, columns, every batch level) steps over everything the smaller ones
// span.  Batches interleaved inside one tensor (C_m[n]p: batch stride below ldc) pass.  Returns -1 if C
// is fine, -2 if ldc is too small, else the batch level whose stride is too small.
int c_overlap(int64_t m, int64_t n, int64_t ldc, int nlevels, const int64_t *stride, const int64_t *count)
{
    struct Dir { int64_t stride, extent; int which; } d[2 + SB_MAX_BATCH_LEVELS];
    int nd = 0;
    if (m > 1) d[nd++] = Dir{1, m, -2};
    if (n > 1) d[nd++] = Dir{ldc, n, -2};
    for (int l = 0; l < nlevels; ++l)
        if (count[l] > 1) d[nd++] = Dir{stride[l], count[l], l};
    for (int a = 1; a < nd; ++a)
        for (int b = a; b > 0 && d[b].stride < d[b - 1].stride; --b) std::swap(d[b], d[b - 1]);
    int64_t span = 0;                      // largest offset reachable with the directions seen so far
    for (int q = 0; q < nd; ++q) {
        if (q > 0 && d[q].stride <= span) return d[q].which;
        span += (d[q].extent - 1) * d[q].stride;
    }
    return -1;
}

int run(sb_dtype dt, const SbArgs &a, hipStream_t stream)
{
    const int kernel = choose(dt, a, g_force_kernel);
    hipError_t err;
    g_last_member = 0;
    switch (kernel) {
    case SB_KERNEL_TINY: err = sb_launch_tiny(dt, a, stream); break;
    case SB_KERNEL_MFMA: err = sb_launch_mfma(dt, a, stream); break;
    case SB_KERNEL_THIN: err = sb_launch_thin(dt, a, stream); break;
    case SB_KERNEL_PANEL: err = sb_launch_panel_bf16(a, stream); break;
    default:             err = sb_launch_generic(dt, a, stream); break;
    }
    g_last_kernel = kernel;
    if (err == hipErrorNoBinaryForGpu) return SB_ERR_NO_DEVICE_CODE;
    return err == hipSuccess ? SB_OK : SB_ERR_LAUNCH + (int)err;
}

}  // namespace

namespace {

// Shared body of sb_gemm2 / sb_gemm_nested: validation, normalisation, launch.  Returns the status in
// sb_gemm_nested's argument numbering; *level receives the batch level a stride or count error refers to.
int gemm_levels(sb_dtype dt, sb_op transA, sb_op transB, int64_t m, int64_t n, int64_t k,
                double alpha, const void *A, int64_t lda, const int64_t *strideA,
                const void *B, int64_t ldb, const int64_t *strideB,
                double beta, void *C, int64_t ldc, const int64_t *strideC,
                int nlevels, const int64_t *batch, void *stream, int *level)
{
    *level = 0;
    if ((int)dt < SB_F64 || (int)dt > SB_BF16) return -1;
    if (!valid_op(transA)) return -2;
    if (!valid_op(transB)) return -3;
    if (m < 0) return -4;
    if (n < 0) return -5;
    if (k < 0) return -6;
    if (nlevels < 0 || nlevels > SB_MAX_BATCH_LEVELS) return -18;
    if (nlevels > 0 && !batch) return -19;
    if (nlevels > 0 && !strideA) return -10;
    if (nlevels > 0 && !strideB) return -13;
    if (nlevels > 0 && !strideC) return -17;
    bool empty = (m == 0 || n == 0);
    for (int l = 0; l < nlevels; ++l) {
        *level = l;
        if (batch[l] < 0) return -19;
        if (batch[l] == 0) empty = true;
    }
    *level = 0;
    if (empty) return SB_OK;
    const bool use_ab = (k > 0 && alpha != 0.0);
    // leading dimensions: at least the number of stored rows (N/T), at least 1 (extended)
    const int64_t rowsA = is_ex(transA) ? 1 : (transA == SB_OP_N ? m : k);
    const int64_t rowsB = is_ex(transB) ? 1 : (transB == SB_OP_N ? k : n);
    // an extended operand reads its stored-column stride from level 0's slot even when there are no levels
    const int64_t sA0 = nlevels > 0 ? strideA[0] : 0, sB0 = nlevels > 0 ? strideB[0] : 0;
    if (use_ab && !A) return -8;
    if (lda < std::max<int64_t>(1, rowsA)) return -9;
    for (int l = 0; l < nlevels; ++l)
        if (strideA[l] < 0) { *level = l; return -10; }
    if (is_ex(transA) && sA0 < 1) return -10;
    if (use_ab && !B) return -11;
    if (ldb < std::max<int64_t>(1, rowsB)) return -12;
    for (int l = 0; l < nlevels; ++l)
        if (strideB[l] < 0) { *level = l; return -13; }
    if (is_ex(transB) && sB0 < 1) return -13;
    if (!C) return -15;
    if (ldc < std::max<int64_t>(1, m)) return -16;
    for (int l = 0; l < nlevels; ++l)
        if (strideC[l] < 0 || (strideC[l] == 0 && batch[l] > 1)) { *level = l; return -17; }
    const int ov = c_overlap(m, n, ldc, nlevels, strideC, batch);
    if (ov == -2) return -16;
    if (ov >= 0) { *level = ov; return -17; }

    SbArgs a;
    std::memset(&a, 0, sizeof(a));
    a.A = A;  a.B = B;  a.C = C;
    a.m = m;  a.n = n;
    a.k = use_ab ? k : 0;                  // alpha == 0: A and B are not read, C = beta*C
    a.alpha = alpha;  a.beta = beta;
    op_strides(transA, lda, sA0, a.rsA, a.csA, a.bsA[0]);
    op_strides(transB, ldb, sB0, a.rsB, a.csB, a.bsB[0]);
    a.ldc = ldc;
    a.bsC[0] = nlevels > 0 ? strideC[0] : 0;
    a.batch0 = nlevels > 0 ? batch[0] : 1;
    a.batch1 = 1;
    a.cnt1 = 1;
    // levels of extent 1 above level 0 drop out; the first remaining one is level 1, the rest fold into its index
    bool have1 = false;
    for (int l = 1; l < nlevels; ++l) {
        if (batch[l] == 1) continue;
        if (!have1) {
            have1 = true;
            a.bsA[1] = strideA[l];  a.bsB[1] = strideB[l];  a.bsC[1] = strideC[l];
            a.cnt1 = batch[l];
        } else {
            a.xcnt[a.nx] = batch[l];
            a.xsA[a.nx] = strideA[l];  a.xsB[a.nx] = strideB[l];  a.xsC[a.nx] = strideC[l];
            ++a.nx;
        }
        if (a.batch1 > (((int64_t)1 << 62) / batch[l])) { *level = l; return -19; }
        a.batch1 *= batch[l];
    }
    return run(dt, a, (hipStream_t)stream);
}

}  // namespace

extern "C" int sb_gemm_nested(sb_dtype dt, sb_op transA, sb_op transB, int64_t m, int64_t n, int64_t k,
                              double alpha, const void *A, int64_t lda, const int64_t *strideA,
                              const void *B, int64_t ldb, const int64_t *strideB,
                              double beta, void *C, int64_t ldc, const int64_t *strideC,
                              int nlevels, const int64_t *batch, void *stream)
{
    int level = 0;
    return gemm_levels(dt, transA, transB, m, n, k, alpha, A, lda, strideA, B, ldb, strideB, beta, C, ldc, strideC,
                       nlevels, batch, stream, &level);
}

extern "C" int sb_gemm2(sb_dtype dt, sb_op transA, sb_op transB, int64_t m, int64_t n, int64_t k,
                        double alpha, const void *A, int64_t lda, int64_t strideA0, int64_t strideA1,
                        const void *B, int64_t ldb, int64_t strideB0, int64_t strideB1,
                        double beta, void *C, int64_t ldc, int64_t strideC0, int64_t strideC1,
                        int64_t batch0, int64_t batch1, void *stream)
{
    const int64_t sA[2] = {strideA0, strideA1}, sB[2] = {strideB0, strideB1}, sC[2] = {strideC0, strideC1};
    const int64_t cnt[2] = {batch0, batch1};
    int level = 0;
    const int rc = gemm_levels(dt, transA, transB, m, n, k, alpha, A, lda, sA, B, ldb, sB, beta, C, ldc, sC, 2, cnt, stream, &level);
    if (rc >= 0) return rc;
    // sb_gemm_nested's argument positions -> sb_gemm2's (each array argument became two scalars)
    switch (-rc) {
    case 10: return -(10 + level);
    case 11: return -12;
    case 12: return -13;
    case 13: return -(14 + level);
    case 15: return -17;
    case 16: return -18;
    case 17: return -(19 + level);
    case 19: return -(21 + level);
    default: return rc;                 // 1 .. 9 keep their positions
    }
}

extern "C" int sb_select_kernel(sb_dtype dt, sb_op transA, sb_op transB, int64_t m, int64_t n, int64_t k,
                                int64_t lda, int64_t strideA, int64_t ldb, int64_t strideB, int64_t ldc,
                                int64_t strideC, int64_t batch)
{
    if ((int)dt < SB_F64 || (int)dt > SB_BF16) return -1;
    if (!valid_op(transA)) return -2;
    if (!valid_op(transB)) return -3;
    if (m < 1) return -4;
    if (n < 1) return -5;
    if (k < 1) return -6;
    if (lda < 1 || strideA < 0) return -7;
    if (ldb < 1 || strideB < 0) return -9;
    if (ldc < m) return -11;
    if (strideC < 0 || (strideC == 0 && batch > 1)) return -12;
    if (batch < 1) return -13;
    switch (c_overlap(m, n, ldc, 1, &strideC, &batch)) {
    case -2: return -11;
    case 0: return -12;
    default: break;
    }
    SbArgs a;
    std::memset(&a, 0, sizeof(a));
    a.m = m;  a.n = n;  a.k = k;
    a.alpha = 1.0;
    op_strides(transA, lda, strideA, a.rsA, a.csA, a.bsA[0]);
    op_strides(transB, ldb, strideB, a.rsB, a.csB, a.bsB[0]);
    a.ldc = ldc;
    a.bsC[0] = strideC;
    a.batch0 = batch;  a.batch1 = 1;
    return choose(dt, a, SB_KERNEL_AUTO);
}

extern "C" int sb_gemm(sb_dtype dt, sb_op transA, sb_op transB, int64_t m, int64_t n, int64_t k,
                       double alpha, const void *A, int64_t lda, int64_t strideA,
                       const void *B, int64_t ldb, int64_t strideB,
                       double beta, void *C, int64_t ldc, int64_t strideC,
                       int64_t batch, void *stream)
{
    int rc = sb_gemm2(dt, transA, transB, m, n, k, alpha, A, lda, strideA, 0, B, ldb, strideB, 0,
                      beta, C, ldc, strideC, 0, batch, 1, stream);
    if (rc >= 0) return rc;
    // renumber sb_gemm2's argument positions to sb_gemm's
    static const int map[24] = {0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 10, 11, 12, 13, 13, 14, 15, 16, 17, 17, 18, 18, 19};
    return -map[-rc];
}

namespace {

// The batch levels of a plan as the launcher sees them.  Two levels whose strides nest in all
// three tensors (stride_outer == stride_inner * count_inner, or both 0) are one level with the
// product of the counts: fewer digits for the kernels to decode, and more problems for the kernels
// that only take two levels.  Whatever remains runs in the same single launch (Listing 2 without
// its host loop).
struct Levels {
    int n;
    int64_t count[SB_MAX_BATCH_LEVELS], sL[SB_MAX_BATCH_LEVELS], sR[SB_MAX_BATCH_LEVELS], sC[SB_MAX_BATCH_LEVELS];
};

Levels merged_levels(const sb_plan &plan)
{
    Levels lv;
    lv.n = plan.nbatch;
    for (int q = 0; q < lv.n; ++q) {
        lv.count[q] = plan.batch[q];
        lv.sL[q] = plan.strideL[q];
        lv.sR[q] = plan.strideR[q];
        lv.sC[q] = plan.strideC[q];
    }
    // level 0 of an extended operation is the operand's unit-stride mode and keeps its own slot
    const int first = (plan.opL > SB_OP_T || plan.opR > SB_OP_T) ? 1 : 0;
    bool changed = true;
    while (changed) {
        changed = false;
        for (int a = first; a < lv.n && !changed; ++a)
            for (int b = first; b < lv.n && !changed; ++b) {
                if (a == b) continue;
                const bool nests = lv.sL[b] == lv.sL[a] * lv.count[a] && lv.sR[b] == lv.sR[a] * lv.count[a] &&
                                   lv.sC[b] == lv.sC[a] * lv.count[a];
                if (!nests) continue;
                lv.count[a] *= lv.count[b];                 // b runs outside a: one level with a's strides
                for (int q = b; q + 1 < lv.n; ++q) {
                    lv.count[q] = lv.count[q + 1];
                    lv.sL[q] = lv.sL[q + 1];
                    lv.sR[q] = lv.sR[q + 1];
                    lv.sC[q] = lv.sC[q + 1];
                }
                --lv.n;
                changed = true;
            }
    }
    return lv;
}

}  // namespace

extern "C" int64_t sb_plan_launches(const sb_plan *plan)
{
    if (!plan || plan->nbatch < 0 || plan->nbatch > SB_MAX_BATCH_LEVELS) return -1;
    return 1;
}

extern "C" int sb_plan_launch(sb_dtype dt, const sb_plan *plan, double alpha, const void *A, const void *B,
                              double beta, void *C, void *stream)
{
    if ((int)dt < SB_F64 || (int)dt > SB_BF16) return -1;
    if (!plan || plan->nbatch < 0 || plan->nbatch > SB_MAX_BATCH_LEVELS) return -2;
    const void *L = plan->left_is_B ? B : A;
    const void *R = plan->left_is_B ? A : B;
    Levels lv = merged_levels(*plan);
    // an extended operand passes its stored-column stride in place of the (implied, unit) level-0 batch stride
    const bool exL = plan->opL > SB_OP_T, exR = plan->opR > SB_OP_T;
    if (lv.n == 0 && (exL || exR)) { lv.n = 1; lv.count[0] = 1; lv.sL[0] = lv.sR[0] = lv.sC[0] = 0; }
    if (exL) lv.sL[0] = plan->exL;
    if (exR) lv.sR[0] = plan->exR;
    int level = 0;
    const int rc = gemm_levels(dt, (sb_op)plan->opL, (sb_op)plan->opR, plan->m, plan->n, plan->k, alpha, L, plan->ldL, lv.sL,
                               R, plan->ldR, lv.sR, beta, C, plan->ldC, lv.sC, lv.n, lv.count, stream, &level);
    if (rc >= 0) return rc;
    // map the failing argument back to this function's: operands 8..13 -> A (4) or B (5), C 15..17 -> 7
    const int p = -rc;
    if (p >= 8 && p <= 13) return (((p <= 10) != (plan->left_is_B != 0)) ? -4 : -5);
    if (p >= 15 && p <= 17) return -7;
    return -2;
}

namespace {

// Iterative algorithms issue the same contraction over and over (only the pointers change), so the
// most recent plan of each thread is kept and reused when every planning input is identical.
struct PlanKey {
    char modes[3][4 * SB_MAX_MODES];
    int64_t dims[3][SB_MAX_MODES], strides[3][SB_MAX_MODES];
    int8_t has_dims[3], has_strides[3];
    int32_t strat;
};

bool fill_key(PlanKey &k, const char *const modes[3], const int64_t *const dims[3], const int64_t *const strides[3], int strat)
{
    std::memset(&k, 0, sizeof(k));
    for (int t = 0; t < 3; ++t) {
        if (!modes[t]) return false;
        const size_t len = std::strlen(modes[t]);
        if (len >= sizeof(k.modes[t])) return false;
        std::memcpy(k.modes[t], modes[t], len);
        int order = 0;
        for (size_t i = 0; i < len; ++i)
            order += (modes[t][i] >= 'a' && modes[t][i] <= 'z') || (modes[t][i] >= 'A' && modes[t][i] <= 'Z');
        if (order > SB_MAX_MODES) return false;
        k.has_dims[t] = dims[t] != nullptr;
        k.has_strides[t] = strides[t] != nullptr;
        for (int j = 0; j < order; ++j) {
            if (dims[t]) k.dims[t][j] = dims[t][j];
            if (strides[t]) k.strides[t][j] = strides[t][j];
        }
    }
    k.strat = strat;
    return true;
}

// A small per-thread cache of recent plans: an iteration such as HOOI cycles through half a dozen
// contractions, each of which finds its plan again as long as every planning input is identical.
struct PlanCache {
    static constexpr int ENTRIES = 8;
    bool valid[ENTRIES] = {};
    PlanKey key[ENTRIES];
    sb_plan plan[ENTRIES];
    int next = 0;                          // round-robin replacement

    const sb_plan *find(const PlanKey &k) const
    {
        for (int e = 0; e < ENTRIES; ++e)
            if (valid[e] && std::memcmp(&key[e], &k, sizeof(k)) == 0) return &plan[e];
        return nullptr;
    }
    void insert(const PlanKey &k, const sb_plan &p)
    {
        std::memcpy(&key[next], &k, sizeof(k));      // byte copy: the keys are compared as bytes, padding included
        plan[next] = p;
        valid[next] = true;
        next = (next + 1) % ENTRIES;
    }
};
thread_local PlanCache g_plan_cache;
thread_local bool g_plan_cache_enabled = true;

}  // namespace

extern "C" int sb_plan_cache_enable(int on)
{
    g_plan_cache_enabled = on != 0;
    return SB_OK;
}

extern "C" int sb_contract(sb_dtype dt, const char *modesA, const char *modesB, const char *modesC,
                           double alpha, const void *A, const int64_t *dimsA, const int64_t *stridesA,
                           const void *B, const int64_t *dimsB, const int64_t *stridesB,
                           double beta, void *C, const int64_t *dimsC, const int64_t *stridesC,
                           sb_strategy strat, void *stream)
{
    if ((int)dt < SB_F64 || (int)dt > SB_BF16) return -1;
    sb_plan planned;
    const sb_plan *plan = nullptr;
    int rc = SB_OK;
    const char *const modes[3] = {modesA, modesB, modesC};
    const int64_t *const dims[3] = {dimsA, dimsB, dimsC};
    const int64_t *const strides[3] = {stridesA, stridesB, stridesC};
    PlanKey key;
    const bool keyed = g_plan_cache_enabled && fill_key(key, modes, dims, strides, (int)strat);
    PlanCache &cache = g_plan_cache;
    if (keyed) plan = cache.find(key);
    if (!plan) {
        rc = sb_contract_plan(modesA, modesB, modesC, dimsA, stridesA, dimsB, stridesB, dimsC, stridesC, strat, &planned);
        if (rc == SB_OK && keyed) cache.insert(key, planned);
        plan = &planned;
    }
    if (rc < 0) {
        // planner argument numbers -> sb_contract argument numbers
        static const int map[12] = {0, 2, 3, 4, 7, 8, 10, 11, 14, 15, 16, 16};
        return -map[-rc];
    }
    if (rc != SB_OK) return rc;
    rc = sb_plan_launch(dt, plan, alpha, A, B, beta, C, stream);
    if (rc < 0) {
        static const int map[9] = {0, 1, 16, 5, 6, 9, 12, 13, 17};
        return -map[-rc];
    }
    return rc;
}

extern "C" int sb_permute(sb_dtype dt, int order, const int64_t *dims, const int *perm, const void *src, void *dst, void *stream)
{
    if ((int)dt < SB_F64 || (int)dt > SB_BF16) return -1;
    if (order < 1 || order > SB_MAX_MODES) return -2;
    if (!dims) return -3;
    if (!perm) return -4;
    bool seen[SB_MAX_MODES] = {};
    int64_t total = 1;
    for (int i = 0; i < order; ++i) {
        if (dims[i] < 0) return -3;
        if (perm[i] < 0 || perm[i] >= order || seen[perm[i]]) return -4;
        seen[perm[i]] = true;
        total *= dims[i];
    }
    if (total == 0) return SB_OK;
    if (!src) return -5;
    if (!dst || dst == src) return -6;
    const hipError_t err = sb_launch_permute(dt == SB_F64 ? 8 : (dt == SB_F32 ? 4 : 2), order, dims, perm, src, dst, (hipStream_t)stream);
    if (err == hipErrorNoBinaryForGpu) return SB_ERR_NO_DEVICE_CODE;
    return err == hipSuccess ? SB_OK : SB_ERR_LAUNCH + (int)err;
}

extern "C" const char *sb_status_string(int status)
{
    if (status == SB_OK) return "success";
    if (status < 0) return "invalid argument (the negated status is the argument's position)";
    switch (status) {
    case SB_ERR_MODES: return "malformed mode string";
    case SB_ERR_CONTRACTION: return "index sets do not form a single-index contraction";
    case SB_ERR_EXTENT: return "inconsistent or negative extent";
    case SB_ERR_STRIDE: return "unusable strides";
    case SB_ERR_ILLEGAL_EVAL: return "the requested evaluation is not legal for this contraction";
    case SB_ERR_NO_DEVICE_CODE: return "no kernel for this device (the library is built for gfx950)";
    default: break;
    }
    if (status >= SB_ERR_LAUNCH) return "kernel launch failed (status - 1000 is the hipError_t)";
    return "unknown status";
}

extern "C" int sb_force_kernel(int kernel_id)
{
    if (kernel_id < SB_KERNEL_AUTO || kernel_id > SB_KERNEL_PANEL) return -1;
    g_force_kernel = kernel_id;
    return SB_OK;
}

extern "C" int sb_last_kernel(void) { return g_last_kernel; }
extern "C" int sb_last_kernel_member(void) { return g_last_member; }
void sb_note_member(int member) { g_last_member = member; }
