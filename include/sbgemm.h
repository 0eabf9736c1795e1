/*
 * sbgemm.h - C ABI of the StridedBatchedGemm / tensor-contraction library for AMD MI355X (gfx950).
 *
 * The library implements the hot path of "Tensor Contractions with Extended BLAS Kernels on CPU
 * and GPU": the StridedBatchedGemm primitive (section III-D, Listing 1) and the mapping of
 * single-index tensor contractions in Einstein notation (section II-B, eq. (1)) onto one
 * flattened GEMM, one StridedBatchedGemm or a nest of them, without copying or transposing
 * any operand (sections III-B to III-F, Tables I and II, Algorithm 2).
 *
 * Conventions common to every entry point
 *   - Storage (section III-B): dense column-major tensors.  Mode i of a tensor has an element
 *     stride ld<i>; a packed tensor has ld<0> = 1 and ld<i> = prod_{j<i} dim<j>.  A matrix
 *     operand is column-major with leading dimension ld: stored element (i,j) is X[i + j*ld].
 *     All sizes, leading dimensions and strides are counted in ELEMENTS and are 64-bit.
 *   - Memory: every tensor pointer is DEVICE memory owned by the caller (for example a torch
 *     tensor's data_ptr()).  The library never allocates, frees, copies or synchronises, and
 *     needs no workspace.  C must not overlap A or B; A and B may alias.
 *   - Streams: `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work; they return before the kernels have run.
 *   - Scalars: alpha and beta are passed as double and converted to the arithmetic type of the
 *     call (double for SB_F64, float for SB_F32 and SB_BF16).
 *   - beta == 0 means C is not read (NaN/Inf in it are overwritten); alpha == 0 or k == 0 give
 *     C = beta*C.  The paper defines the beta term in eq. (1) but only ever calls with beta = 0;
 *     this is the BLAS convention.
 *   - Errors: functions return an int.  0 = SB_OK.  A negative value -i means the i-th argument
 *     (1-based, in declaration order) is invalid; nothing was launched.  Positive values are the
 *     SB_ERR_* codes below.  Nothing is printed and nothing aborts.
 *   - Quick returns: batch == 0, m == 0 or n == 0 return SB_OK without touching memory.
 */
#ifndef SBGEMM_H
#define SBGEMM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Operation applied to a stored matrix operand.
 * SB_OP_N / SB_OP_T: the stored matrix or its transpose, as in GEMM.
 * SB_OP_EX_N / SB_OP_EX_T: the "extended" operations proposed in section III-E for the
 * exceptional cases of Table II, where the batched mode is the FIRST (unit-stride) mode of the
 * operand.  The batch stride of such an operand is 1 by definition, so its two stride arguments
 * carry the strides of the other two modes in row-column order of the stored matrix:
 * `ld` = stride between stored rows, `stride` = stride between stored columns; stored element
 * (i,j) of batch b is X[b + i*ld + j*stride].  EX_T uses the transpose of that stored matrix. */
typedef enum { SB_OP_N = 0, SB_OP_T = 1, SB_OP_EX_N = 2, SB_OP_EX_T = 3 } sb_op;

/* Element type of A, B and C.  SB_BF16: bf16 inputs and output, fp32 products and accumulation,
 * output rounded to nearest-even. */
typedef enum { SB_F64 = 0, SB_F32 = 1, SB_BF16 = 2 } sb_dtype;

/* How sb_contract chooses among the legal evaluations of a contraction (section IV-D).
 * Mode strings that carry [ ] or ( ) annotations select the evaluation themselves and need SB_AUTO. */
typedef enum {
    SB_AUTO = 0,       /* flatten whenever possible; GEMM over the largest legal mode, batch the rest */
    SB_FLATTEN = 1,    /* a single flattened GEMM, or SB_ERR_ILLEGAL_EVAL if flattening cannot remove every batch mode */
    SB_BATCH_LAST = 2, /* no flattening; GEMM columns = 2nd mode of C, every later mode batched ("[p]") */
    SB_BATCH_MID = 3,  /* no flattening; GEMM columns = last mode of C, the modes between batched ("[n]") */
    SB_NESTED = 4,     /* no flattening; GEMM over the largest legal mode, all other free modes batched */
    SB_LEVEL2 = 5      /* batched matrix-vector evaluation (Table II's second kernel of the exceptional rows) */
} sb_strategy;

enum {
    SB_OK = 0,
    SB_ERR_MODES = 1,        /* malformed mode string: bad character, unbalanced [ ] ( ), repeated index, too many modes */
    SB_ERR_CONTRACTION = 2,  /* index sets violate eq. (1), or not exactly one contracted index */
    SB_ERR_EXTENT = 3,       /* an index has different extents in two tensors, or a negative extent */
    SB_ERR_STRIDE = 4,       /* strides unusable: not positive, or matrix columns / batches of C overlap */
    SB_ERR_ILLEGAL_EVAL = 5, /* the requested evaluation breaks rules 1-4 of section III-B or does not exist */
    SB_ERR_NO_DEVICE_CODE = 6, /* the library holds no kernel for this device (not gfx950) */
    SB_ERR_LAUNCH = 1000     /* SB_ERR_LAUNCH + hipError_t of a failed kernel launch */
};

/*
 * StridedBatchedGemm (section III-D, Listing 1):
 *     C_p = alpha * opA(A_p) * opB(B_p) + beta * C_p,   X_p = X + p*strideX,   p = 0 .. batch-1
 * opA(A_p) is m x k, opB(B_p) is k x n, C_p is m x n.  lda/ldb/ldc are the usual leading
 * dimensions ("stride between columns"), strideA/B/C the paper's "leading order" loa/lob/loc
 * ("stride between matrices of the batch").
 *   - strideA or strideB may be 0 (the operand is shared by all batches, Listing 2).
 *   - strideC may be smaller than ldc*n (batches interleaved inside one tensor, as in the
 *     C_m[n]p evaluations of Table II), but two batches must not share an element: strideC == 0
 *     with batch > 1 is rejected (-17), and so is any C whose rows, columns and batches, sorted by
 *     stride, do not each step over everything the smaller strides span (the argument named is
 *     the stride that is too small: -16 for ldc, -17 for strideC).
 *   - ld >= max(1, stored rows) is required for SB_OP_N / SB_OP_T operands and for C.
 *   - For SB_OP_EX_* see sb_op.
 * Argument numbers for the error code: dt=1 transA=2 transB=3 m=4 n=5 k=6 alpha=7 A=8 lda=9
 * strideA=10 B=11 ldb=12 strideB=13 beta=14 C=15 ldc=16 strideC=17 batch=18 stream=19.
 */
int sb_gemm(sb_dtype dt, sb_op transA, sb_op transB, int64_t m, int64_t n, int64_t k,
            double alpha, const void *A, int64_t lda, int64_t strideA,
            const void *B, int64_t ldb, int64_t strideB,
            double beta, void *C, int64_t ldc, int64_t strideC,
            int64_t batch, void *stream);

/*
 * Nested batching in ONE launch (section III-F, Listing 2): two batch levels,
 *     X_{p,q} = X + p*strideX0 + q*strideX1,   p < batch0,  q < batch1.
 * Equivalent to `for q: sb_gemm(..., A + q*strideA1, ..., batch0)`.  For an SB_OP_EX_* operand
 * strideX0 is the stored-column stride (see sb_op) and its level-0 batch stride is 1.
 * Distinct (p,q) must address disjoint C_pq (checked as for sb_gemm: -18 ldc, -19 strideC0, -20 strideC1).
 * Argument numbers: dt=1 transA=2 transB=3 m=4 n=5 k=6 alpha=7 A=8 lda=9 strideA0=10 strideA1=11
 * B=12 ldb=13 strideB0=14 strideB1=15 beta=16 C=17 ldc=18 strideC0=19 strideC1=20 batch0=21
 * batch1=22 stream=23.
 */
int sb_gemm2(sb_dtype dt, sb_op transA, sb_op transB, int64_t m, int64_t n, int64_t k,
             double alpha, const void *A, int64_t lda, int64_t strideA0, int64_t strideA1,
             const void *B, int64_t ldb, int64_t strideB0, int64_t strideB1,
             double beta, void *C, int64_t ldc, int64_t strideC0, int64_t strideC1,
             int64_t batch0, int64_t batch1, void *stream);

/*
 * Nested batching to any depth in ONE launch (section III-F: Listing 2 with as many loops as the
 * contraction has batched modes, and none of them on the host): nlevels <= SB_MAX_BATCH_LEVELS levels,
 *     X_{p0,p1,..} = X + sum_l p_l * strideX[l],   p_l < batch[l],   level 0 innermost.
 * strideA / strideB / strideC / batch are HOST arrays of nlevels entries (NULL allowed when nlevels
 * is 0), read before the call returns.  For an SB_OP_EX_* operand strideX[0] is the stored-column
 * stride (see sb_op) and its level-0 batch stride is 1.  Distinct index tuples must address disjoint
 * C (checked as for sb_gemm).  Every kernel family takes two levels directly; deeper levels are a
 * mixed-radix decode of the level-1 index inside the tiled and small-matrix kernels (the level-2
 * kernels of SB_KERNEL_THIN and the panel kernel of SB_KERNEL_PANEL leave such nests to them).
 * Argument numbers: dt=1 transA=2 transB=3 m=4 n=5 k=6 alpha=7 A=8 lda=9 strideA=10 B=11 ldb=12
 * strideB=13 beta=14 C=15 ldc=16 strideC=17 nlevels=18 batch=19 stream=20.
 */
#define SB_MAX_MODES 8          /* largest tensor order accepted */
#define SB_MAX_BATCH_LEVELS 8   /* most batch levels of one call; all of them run inside one launch */
int sb_gemm_nested(sb_dtype dt, sb_op transA, sb_op transB, int64_t m, int64_t n, int64_t k,
                   double alpha, const void *A, int64_t lda, const int64_t *strideA,
                   const void *B, int64_t ldb, const int64_t *strideB,
                   double beta, void *C, int64_t ldc, const int64_t *strideC,
                   int nlevels, const int64_t *batch, void *stream);

/* The evaluation chosen for a contraction: the arguments of one (nested) StridedBatchedGemm. */
typedef struct {
    int32_t nbatch;       /* number of batched modes: 0 = one flattened GEMM, 1 = one StridedBatchedGemm, >1 = nested */
    int32_t exceptional;  /* 1 if the evaluation needs an extended operation or a matrix-vector form (section III-E) */
    int32_t left_is_B;    /* 0: tensor A feeds the first GEMM operand and B the second; 1: the reverse (rule 4, C = B.. A..) */
    int32_t opL, opR;     /* sb_op of the first / second GEMM operand */
    int64_t m, n, k;      /* GEMM extents (products of extents for flattened modes) */
    int64_t ldL, ldR, ldC;    /* leading dimensions; for an SB_OP_EX_* operand: its stored-row stride */
    int64_t exL, exR;         /* stored-column stride of an SB_OP_EX_* operand, else 0 */
    int64_t batch[SB_MAX_BATCH_LEVELS];    /* extent of each batched mode, level 0 first */
    int64_t strideL[SB_MAX_BATCH_LEVELS];  /* element stride of that mode in each operand (0 = operand lacks it) */
    int64_t strideR[SB_MAX_BATCH_LEVELS];
    int64_t strideC[SB_MAX_BATCH_LEVELS];
    char notation[192];   /* the evaluation in the paper's notation, e.g. "C_m[n]p = B_k[n]m^T A_pk^T" */
} sb_plan;

/*
 * Contraction planner (host only, touches no device): maps
 *     C_modesC = alpha * A_modesA * B_modesB + beta * C_modesC            (eq. (1))
 * with exactly one contracted index onto StridedBatchedGemm arguments, following the notation
 * rules of section III-B, the case analysis behind Table II and the priorities of section IV-D /
 * Algorithm 2.
 *   - modesX: one letter per mode, first mode first ("knp").  The strings may be annotated in the
 *     paper's notation to demand a specific evaluation: "[p]" batches mode p, "(np)" flattens
 *     modes n and p, e.g. ("mk", "k[n]p", "m[n]p") or ("mk", "k(np)", "m(np)").  An annotation
 *     given on one tensor applies to the same indices of the others.  Annotated strings need
 *     strat == SB_AUTO.
 *   - dimsX: extent of each mode of X, in X's mode order.  dimsC may be NULL (derived from A, B).
 *   - stridesX: element stride of each mode, or NULL for packed storage.
 * Operand placement follows rule 4: the tensor holding C's first mode becomes the first GEMM
 * operand; transposes are read off from which mode of an operand has unit stride; a batched mode
 * may not be an operand's unit-stride mode (rule 1) unless an extended operation is used;
 * flattening needs ld<j> = ld<i>*dim<i> and the same modes in the same order on both sides
 * (rules 2, 3).
 * Argument numbers: modesA=1 modesB=2 modesC=3 dimsA=4 stridesA=5 dimsB=6 stridesB=7 dimsC=8
 * stridesC=9 strat=10 out=11.
 */
int sb_contract_plan(const char *modesA, const char *modesB, const char *modesC,
                     const int64_t *dimsA, const int64_t *stridesA,
                     const int64_t *dimsB, const int64_t *stridesB,
                     const int64_t *dimsC, const int64_t *stridesC,
                     sb_strategy strat, sb_plan *out);

/*
 * Tensor contraction on device tensors: plans as sb_contract_plan does, then launches the plan:
 * ONE launch whatever the number of batched modes (the loops of Listing 2 all run inside the
 * kernel).  No operand is copied or transposed.
 * Argument numbers: dt=1 modesA=2 modesB=3 modesC=4 alpha=5 A=6 dimsA=7 stridesA=8 B=9 dimsB=10
 * stridesB=11 beta=12 C=13 dimsC=14 stridesC=15 strat=16 stream=17.
 */
int sb_contract(sb_dtype dt, const char *modesA, const char *modesB, const char *modesC,
                double alpha, const void *A, const int64_t *dimsA, const int64_t *stridesA,
                const void *B, const int64_t *dimsB, const int64_t *stridesB,
                double beta, void *C, const int64_t *dimsC, const int64_t *stridesC,
                sb_strategy strat, void *stream);

/* sb_contract keeps the plans of the calling thread's eight most recent distinct contractions
 * (mode strings, extents, strides and strategy all equal: pointers and scalars may differ) and
 * skips the planner when one of them comes again.  sb_plan_cache_enable(0) switches that off for
 * the calling thread (benchmarks that want the planner inside the timed call), (1) on again. */
int sb_plan_cache_enable(int on);

/* Launch a plan produced by sb_contract_plan on the tensors it was planned for (device pointers
 * A, B, C of the ORIGINAL contraction; the plan knows which one feeds which GEMM slot).
 * Argument numbers: dt=1 plan=2 alpha=3 A=4 B=5 beta=6 C=7 stream=8. */
int sb_plan_launch(sb_dtype dt, const sb_plan *plan, double alpha, const void *A, const void *B,
                   double beta, void *C, void *stream);

/* Host only: the number of kernel launches sb_plan_launch issues for this plan: always 1 (levels whose
 * strides nest in all three tensors are merged, the others are decoded inside the kernel).  -1 for an
 * invalid plan. */
int64_t sb_plan_launches(const sb_plan *plan);

/*
 * Out-of-place mode permutation of a packed column-major device tensor: dst mode j is src mode
 * perm[j] (dims: extents of src).  This is the explicit copy of the CONVENTIONAL evaluation of a
 * contraction (section II-D: permute the operands into matricised form, one GEMM, permute the
 * result back), which the contraction entry points above exist to avoid and never call; it is
 * exported so that a benchmark can price that copy next to the same GEMM code.  src and dst must
 * not overlap.  Argument numbers: dt=1 order=2 dims=3 perm=4 src=5 dst=6 stream=7.
 */
int sb_permute(sb_dtype dt, int order, const int64_t *dims, const int *perm, const void *src, void *dst, void *stream);

/* Static text for a status code returned by any function above. */
const char *sb_status_string(int status);

/* Kernel families behind sb_gemm (diagnostics: tests and the benchmark use these to make sure the
 * intended path ran).  sb_force_kernel(id) makes later calls OF THE CALLING THREAD use that family
 * whenever it takes the problem (SB_KERNEL_AUTO restores the selector); sb_last_kernel() is the
 * family of the calling thread's most recent launch (-1 before any).  Both are per host thread.
 * What each family takes when forced (anything else falls to SB_KERNEL_GENERIC):
 *   SB_KERNEL_GENERIC  every problem the entry points accept;
 *   SB_KERNEL_THIN     1 <= min(m, n) <= 4, any operation and element type;
 *   SB_KERNEL_TINY     SB_F64 / SB_F32, m <= 32 and n <= 32, k >= 1, operations N / T;
 *   SB_KERNEL_MFMA     k >= 1, operations N / T in every element type; an extended operation on ONE
 *                      operand (the other N / T with batch stride 0 at level 0) in every element type
 *                      when batch0 >= 8 and op(X)'s free extent is >= 8 for the extended operand and
 *                      >= 16 for the other (first operand: m >= 8, n >= 16; second: n >= 8, m >= 16);
 *   SB_KERNEL_PANEL    SB_BF16 with 1 <= k <= 128, operations N / T (whole-k operand panels in LDS: the
 *                      selector takes it when C has at least 4 x 4 blocks of 64 x 64 -- counting, on
 *                      each side, the batch levels that move only that side's operand -- and at least
 *                      128 blocks of 256 x 256; smaller problems run on SB_KERNEL_MFMA's 64 x 64 tiles,
 *                      which fetch an operand panel per 64 x 64 block instead of per four). */
enum { SB_KERNEL_AUTO = -1, SB_KERNEL_GENERIC = 0, SB_KERNEL_TINY = 1, SB_KERNEL_MFMA = 2, SB_KERNEL_THIN = 3, SB_KERNEL_PANEL = 4 };
int sb_force_kernel(int kernel_id);
int sb_last_kernel(void);
/* Which member of its family the calling thread's most recent launch ran, for the families whose
 * members differ in more than tile size (0 for the others): tests use it to make sure that a problem
 * built for a member still reaches it.
 *   SB_KERNEL_PANEL: SB_MEMBER_PANEL_4X4 (4 x 4 panels per workgroup, staged through registers: any shape)
 *                    or SB_MEMBER_PANEL_WIDE (2 x 8 panels straight into LDS: k == 128, beta == 0, whole
 *                    64-wide panels in whole blocks, every address 16-byte aligned);
 *   SB_KERNEL_TINY:  SB_MEMBER_TINY_WHOLE (one wave per C_p) or SB_MEMBER_TINY_BLOCKS (a batch of at most
 *                    1024 / (blocks per C_p) problems with m or n == 32 run as independent 16 x 16 blocks);
 *   SB_KERNEL_MFMA, extended operation only: SB_MEMBER_MFMA_EX_BRICK (bricks of 16 batches x 16 rows, staged
 *                    through registers: any shape), SB_MEMBER_MFMA_EX_SMALL (quarter-size tiles when there are
 *                    fewer than 128 large ones; SB_F32 / SB_F64) or SB_MEMBER_MFMA_EX_DMA (SB_F32 / SB_F64, whole
 *                    bricks -- batch a multiple of 16, the extended operand's free extent of 16, the other's of
 *                    64, k of 64 bytes -- loaded straight into LDS; operands 16-byte aligned, strides multiples
 *                    of 16 bytes). */
enum { SB_MEMBER_PANEL_4X4 = 1, SB_MEMBER_PANEL_WIDE = 2, SB_MEMBER_TINY_WHOLE = 1, SB_MEMBER_TINY_BLOCKS = 2,
       SB_MEMBER_MFMA_EX_BRICK = 1, SB_MEMBER_MFMA_EX_SMALL = 2, SB_MEMBER_MFMA_EX_DMA = 3 };
int sb_last_kernel_member(void);

/* Host only: the kernel family the selector sends an sb_gemm problem to (sizes, operations and
 * strides as for sb_gemm, all of m, n, k, batch at least 1; no pointers: the family depends on the
 * shape only; no alignment beyond that of the elements is ever required of the operands).  Negative: -i = i-th argument
 * invalid (C is checked as in sb_gemm: -11 ldc, -12 strideC).  Ignores sb_force_kernel.
 * Argument numbers: dt=1 transA=2 transB=3 m=4 n=5 k=6 lda=7 strideA=8 ldb=9 strideB=10 ldc=11 strideC=12 batch=13. */
int sb_select_kernel(sb_dtype dt, sb_op transA, sb_op transB, int64_t m, int64_t n, int64_t k,
                     int64_t lda, int64_t strideA, int64_t ldb, int64_t strideB, int64_t ldc,
                     int64_t strideC, int64_t batch);

/* Diagnostics for benchmarks: enqueue a kernel that only issues the MFMA instruction the kernels of
 * element type dt are built on (4 independent accumulators per wave, 16 waves per compute unit),
 * `iterations` rounds (a multiple of 16); *flops receives the floating-point operations it performs, so that
 * flops / measured time is the matrix-core rate this device sustains.  scratch: device memory of at
 * least 2 MiB that the kernel overwrites.
 * Argument numbers: dt=1 iterations=2 scratch=3 scratch_bytes=4 stream=5 flops=6. */
int sb_probe_mfma(sb_dtype dt, int iterations, void *scratch, int64_t scratch_bytes, void *stream, double *flops);

#ifdef __cplusplus
}
#endif
#endif /* SBGEMM_H */
