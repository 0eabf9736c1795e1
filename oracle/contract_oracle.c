/*
 * CPU oracle for tensor contractions and StridedBatchedGemm.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the GPU library and must never be called from the product path; only
 * the test-suite, the smoke check and the benchmark's CPU-baseline leg use it.
 *
 * What it computes
 *   oracle_contract      : the general contraction of the paper's eq. (1)
 *                          (section II-B),  C_C = alpha * A_A * B_B + beta * C_C
 *                          with Einstein summation over the indices common to
 *                          A and B, evaluated element by element as a plain
 *                          nested loop.  Element addresses follow the
 *                          column-major strided storage model of section III-B:
 *                          element (i0,i1,...) of X lives at X[sum_j i_j*ld<j>].
 *   oracle_contract_at   : the same sum for a caller-chosen list of output
 *                          multi-indices only (for spot checks at sizes where
 *                          the full loop would take too long).
 *   oracle_sb_gemm       : the StridedBatchedGemm definition of Listing 1
 *                          (section III-D): for every p < batch a textbook
 *                          GEMM on A + p*loa, B + p*lob, C + p*loc.
 *
 * Precision: all tensors are passed as fp64 (fp32 and bf16 values are exactly
 * representable in fp64).  Sums are accumulated in long double when `wide` is
 * non-zero (used for fp64 parity, so that the oracle's own rounding error is
 * far below the 1e-12 gate) and in double otherwise.
 *
 * Readings where the paper is silent:
 *   - beta == 0 means "C is not read": the result is alpha*sum even if the old
 *     C holds NaN/Inf (BLAS convention; every call printed in the paper uses
 *     beta = 0).
 *   - an empty contracted range (extent 0) gives sum = 0.
 *
 * Return value: 0 on success, a negative number naming the first bad argument
 * group otherwise (-1 modes of A, -2 modes of B, -3 modes of C, -4 extents).
 */
#include <stdint.h>
#include <string.h>

#define ORACLE_MAX_LABELS 32

typedef struct {
    int nlabels;
    char label[ORACLE_MAX_LABELS];
    int64_t extent[ORACLE_MAX_LABELS];
    /* stride of every label in each tensor, 0 if the tensor lacks it */
    int64_t sA[ORACLE_MAX_LABELS], sB[ORACLE_MAX_LABELS], sC[ORACLE_MAX_LABELS];
    int inA[ORACLE_MAX_LABELS], inB[ORACLE_MAX_LABELS], inC[ORACLE_MAX_LABELS];
    /* label numbers of C's modes in C's order, and of the contracted labels */
    int nfree, free_[ORACLE_MAX_LABELS];
    int nsum, sum_[ORACLE_MAX_LABELS];
} spec_t;

static int find_label(const spec_t *s, char c)
{
    for (int i = 0; i < s->nlabels; ++i)
        if (s->label[i] == c) return i;
    return -1;
}

/* Register the modes of one tensor; `which` is 0,1,2 for A,B,C. */
static int add_tensor(spec_t *s, int which, const char *modes,
                      const int64_t *dims, const int64_t *ld)
{
    int n = (int)strlen(modes);
    for (int j = 0; j < n; ++j) {
        for (int j2 = 0; j2 < j; ++j2)
            if (modes[j2] == modes[j]) return -1;          /* repeated index in one tensor */
        int id = find_label(s, modes[j]);
        if (id < 0) {
            if (s->nlabels == ORACLE_MAX_LABELS) return -1;
            id = s->nlabels++;
            s->label[id] = modes[j];
            s->extent[id] = dims[j];
            s->sA[id] = s->sB[id] = s->sC[id] = 0;
            s->inA[id] = s->inB[id] = s->inC[id] = 0;
        } else if (s->extent[id] != dims[j]) {
            return -4;                                      /* same index, different extent */
        }
        if (dims[j] < 0) return -4;
        if (which == 0) { s->sA[id] = ld[j]; s->inA[id] = 1; }
        if (which == 1) { s->sB[id] = ld[j]; s->inB[id] = 1; }
        if (which == 2) { s->sC[id] = ld[j]; s->inC[id] = 1; }
    }
    return 0;
}

static int build_spec(spec_t *s,
                      const char *mA, const int64_t *dA, const int64_t *lA,
                      const char *mB, const int64_t *dB, const int64_t *lB,
                      const char *mC, const int64_t *dC, const int64_t *lC)
{
    int rc;
    s->nlabels = 0;
    if ((rc = add_tensor(s, 0, mA, dA, lA)) != 0) return rc == -4 ? -4 : -1;
    if ((rc = add_tensor(s, 1, mB, dB, lB)) != 0) return rc == -4 ? -4 : -2;
    if ((rc = add_tensor(s, 2, mC, dC, lC)) != 0) return rc == -4 ? -4 : -3;
    /* eq. (1): the modes of C are exactly the indices that occur in one of A, B
       but not in both; the indices in both are summed. */
    s->nfree = 0;
    s->nsum = 0;
    for (int i = 0; i < s->nlabels; ++i) {
        int both = s->inA[i] && s->inB[i];
        int one = (s->inA[i] || s->inB[i]) && !both;
        if (both && s->inC[i]) return -3;
        if (one && !s->inC[i]) return -3;
        if (!s->inA[i] && !s->inB[i]) return -3;            /* index only in C */
        if (both) s->sum_[s->nsum++] = i;
    }
    int nC = (int)strlen(mC);
    for (int j = 0; j < nC; ++j) s->free_[s->nfree++] = find_label(s, mC[j]);
    return 0;
}

/* The inner sum of eq. (1) for one fixed assignment of the free indices. */
static long double sum_wide(const spec_t *s, const double *A, const double *B,
                            int64_t baseA, int64_t baseB)
{
    int64_t idx[ORACLE_MAX_LABELS];
    int64_t total = 1;
    for (int j = 0; j < s->nsum; ++j) { idx[j] = 0; total *= s->extent[s->sum_[j]]; }
    long double acc = 0.0L;
    for (int64_t t = 0; t < total; ++t) {
        int64_t oa = baseA, ob = baseB;
        for (int j = 0; j < s->nsum; ++j) {
            oa += idx[j] * s->sA[s->sum_[j]];
            ob += idx[j] * s->sB[s->sum_[j]];
        }
        acc += (long double)A[oa] * (long double)B[ob];
        for (int j = 0; j < s->nsum; ++j) {                 /* odometer over summed indices */
            if (++idx[j] < s->extent[s->sum_[j]]) break;
            idx[j] = 0;
        }
    }
    return acc;
}

static double sum_double(const spec_t *s, const double *A, const double *B,
                         int64_t baseA, int64_t baseB)
{
    int64_t idx[ORACLE_MAX_LABELS];
    int64_t total = 1;
    for (int j = 0; j < s->nsum; ++j) { idx[j] = 0; total *= s->extent[s->sum_[j]]; }
    double acc = 0.0;
    for (int64_t t = 0; t < total; ++t) {
        int64_t oa = baseA, ob = baseB;
        for (int j = 0; j < s->nsum; ++j) {
            oa += idx[j] * s->sA[s->sum_[j]];
            ob += idx[j] * s->sB[s->sum_[j]];
        }
        acc += A[oa] * B[ob];
        for (int j = 0; j < s->nsum; ++j) {
            if (++idx[j] < s->extent[s->sum_[j]]) break;
            idx[j] = 0;
        }
    }
    return acc;
}

/* One output element: cidx[j] is the value of C's j-th mode. */
static double one_element(const spec_t *s, const double *A, const double *B,
                          const double *C, const int64_t *cidx,
                          double alpha, double beta, int wide, int64_t *offC_out)
{
    int64_t oa = 0, ob = 0, oc = 0;
    for (int j = 0; j < s->nfree; ++j) {
        int id = s->free_[j];
        oa += cidx[j] * s->sA[id];
        ob += cidx[j] * s->sB[id];
        oc += cidx[j] * s->sC[id];
    }
    *offC_out = oc;
    if (wide) {
        long double v = (long double)alpha * sum_wide(s, A, B, oa, ob);
        if (beta != 0.0) v += (long double)beta * (long double)C[oc];
        return (double)v;
    } else {
        double v = alpha * sum_double(s, A, B, oa, ob);
        if (beta != 0.0) v += beta * C[oc];
        return v;
    }
}

int oracle_contract(const char *modesA, const int64_t *dimsA, const int64_t *ldA, const double *A,
                    const char *modesB, const int64_t *dimsB, const int64_t *ldB, const double *B,
                    const char *modesC, const int64_t *dimsC, const int64_t *ldC, double *C,
                    double alpha, double beta, int wide)
{
    spec_t s;
    int rc = build_spec(&s, modesA, dimsA, ldA, modesB, dimsB, ldB, modesC, dimsC, ldC);
    if (rc) return rc;
    int64_t total = 1;
    for (int j = 0; j < s.nfree; ++j) total *= s.extent[s.free_[j]];
    /* every output element is independent: split them over the host threads */
    #pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < total; ++t) {
        int64_t cidx[ORACLE_MAX_LABELS];
        int64_t rem = t;
        for (int j = 0; j < s.nfree; ++j) {                 /* first mode of C runs fastest */
            int64_t e = s.extent[s.free_[j]];
            cidx[j] = rem % e;
            rem /= e;
        }
        int64_t oc;
        double v = one_element(&s, A, B, C, cidx, alpha, beta, wide, &oc);
        C[oc] = v;
    }
    return 0;
}

/* out[i] = value of eq. (1) at the output multi-index cidx[i*order(C) ...]; C is only read. */
int oracle_contract_at(const char *modesA, const int64_t *dimsA, const int64_t *ldA, const double *A,
                       const char *modesB, const int64_t *dimsB, const int64_t *ldB, const double *B,
                       const char *modesC, const int64_t *dimsC, const int64_t *ldC, const double *C,
                       double alpha, double beta, int wide,
                       int64_t nsamples, const int64_t *cidx, double *out)
{
    spec_t s;
    int rc = build_spec(&s, modesA, dimsA, ldA, modesB, dimsB, ldB, modesC, dimsC, ldC);
    if (rc) return rc;
    for (int64_t i = 0; i < nsamples; ++i)
        for (int j = 0; j < s.nfree; ++j)
            if (cidx[i * s.nfree + j] < 0 || cidx[i * s.nfree + j] >= s.extent[s.free_[j]]) return -4;
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nsamples; ++i) {
        int64_t oc;
        out[i] = one_element(&s, A, B, C, cidx + i * s.nfree, alpha, beta, wide, &oc);
    }
    return 0;
}

/*
 * Listing 1: C_p = alpha * opA(A_p) * opB(B_p) + beta * C_p with X_p = X + p*lox.
 * opX is 'N' (the stored matrix) or 'T' (its transpose); matrices are
 * column-major with leading dimension ldx, so stored element (i,j) is X[i + j*ldx].
 */
int oracle_sb_gemm(char opA, char opB, int64_t m, int64_t n, int64_t k,
                   double alpha, const double *A, int64_t lda, int64_t loa,
                   const double *B, int64_t ldb, int64_t lob,
                   double beta, double *C, int64_t ldc, int64_t loc,
                   int64_t batch, int wide)
{
    if (opA != 'N' && opA != 'T') return -1;
    if (opB != 'N' && opB != 'T') return -2;
    if (m < 0 || n < 0 || k < 0 || batch < 0) return -4;
    #pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < batch; ++p) {
        const double *Ap = A + p * loa;
        const double *Bp = B + p * lob;
        double *Cp = C + p * loc;
        for (int64_t j = 0; j < n; ++j) {
            for (int64_t i = 0; i < m; ++i) {
                long double accw = 0.0L;
                double accd = 0.0;
                for (int64_t l = 0; l < k; ++l) {
                    double a = (opA == 'N') ? Ap[i + l * lda] : Ap[l + i * lda];
                    double b = (opB == 'N') ? Bp[l + j * ldb] : Bp[j + l * ldb];
                    if (wide) accw += (long double)a * (long double)b;
                    else      accd += a * b;
                }
                if (wide) {
                    long double v = (long double)alpha * accw;
                    if (beta != 0.0) v += (long double)beta * (long double)Cp[i + j * ldc];
                    Cp[i + j * ldc] = (double)v;
                } else {
                    double v = alpha * accd;
                    if (beta != 0.0) v += beta * Cp[i + j * ldc];
                    Cp[i + j * ldc] = v;
                }
            }
        }
    }
    return 0;
}
