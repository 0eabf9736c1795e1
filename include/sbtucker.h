/*
 * sbtucker.h - C ABI of the Tucker decomposition by higher-order orthogonal iteration (HOOI),
 * the application study of "Tensor Contractions with Extended BLAS Kernels on CPU and GPU"
 * (section II-C, Algorithm 1; measured in section IV-C), built on the contraction entry points of
 * sbgemm.h.  Conventions (column-major device tensors, sizes in elements, stream as void*,
 * status codes, nothing allocated or synchronised by the library) are those of sbgemm.h.
 *
 * T_mnp ~ G_ijk A_mi B_nj C_pk with orthonormal columns in A (m x i), B (n x j), C (p x k).
 * Every contraction of Algorithm 1 (steps 4, 6, 8, 11) runs through sb_contract without copying
 * or transposing T.  "The r leading left singular vectors of Y_(mode)" are computed as the
 * leading eigenvectors of the Gram matrix of the shorter side of the unfolding (formed by
 * sb_gemm, diagonalised by Jacobi rotations on the device) mapped back through Y; they are
 * defined up to sign, so only A A^T, B B^T, C C^T and G x1 A x2 B x3 C are unique.
 */
#ifndef SBTUCKER_H
#define SBTUCKER_H

#include <stdint.h>

#include "sbgemm.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Bytes of device workspace sb_tucker_hooi needs for these sizes (dt = SB_F32 or SB_F64).
 * with_init != 0 includes the Gram matrices of T's own unfoldings (m x m, n x n, p x p).
 * Argument numbers: dt=1 m=2 n=3 p=4 i=5 j=6 k=7 with_init=8 bytes=9. */
int sb_tucker_workspace(sb_dtype dt, int64_t m, int64_t n, int64_t p, int64_t i, int64_t j, int64_t k,
                        int with_init, int64_t *bytes);

/*
 * Algorithm 1 for a third-order tensor T (m x n x p, packed column-major) and core size i x j x k
 * (1 <= i <= min(m, j*k), likewise for j and k).
 *   init != 0: step 2, the factors start as the leading left singular vectors of T_(1), T_(2), T_(3);
 *   init == 0: A, B, C hold the caller's starting factors (orthonormal columns).
 *   iterations: number of passes over steps 4-9 (0 is allowed).
 * On completion (of the stream) A, B, C hold the factors and G (i x j x k, packed) the core of
 * step 11.  workspace: device memory of at least sb_tucker_workspace(...) bytes, 256-byte aligned,
 * contents irrelevant before and after.  Everything is enqueued on `stream`; no host
 * synchronisation happens, so the call can be captured in a graph once the kernels are warm.
 * Argument numbers: dt=1 T=2 m=3 n=4 p=5 i=6 j=7 k=8 iterations=9 init=10 A=11 B=12 C=13 G=14
 * workspace=15 workspace_bytes=16 stream=17.
 */
int sb_tucker_hooi(sb_dtype dt, const void *T, int64_t m, int64_t n, int64_t p, int64_t i, int64_t j, int64_t k,
                   int iterations, int init, void *A, void *B, void *C, void *G,
                   void *workspace, int64_t workspace_bytes, void *stream);

/*
 * The symmetric eigensolver used inside (parallel-ordered two-sided Jacobi), exposed for testing:
 * S (n x n, symmetric, packed column-major, n <= 4096) is destroyed; on completion lambda holds the
 * eigenvalues in descending order and V (n x n) the matching eigenvectors as columns.
 * workspace: device memory of at least sb_sym_eig_workspace(...) bytes, 256-byte aligned.
 * sweeps <= 0 selects the default for dt.
 * Argument numbers: dt=1 n=2 S=3 V=4 lambda=5 sweeps=6 workspace=7 workspace_bytes=8 stream=9.
 */
int sb_sym_eig_workspace(sb_dtype dt, int64_t n, int64_t *bytes);
int sb_sym_eig(sb_dtype dt, int64_t n, void *S, void *V, void *lambda, int sweeps,
               void *workspace, int64_t workspace_bytes, void *stream);

/*
 * sb_sym_eig for callers that cannot allocate device memory or pass a workspace: code running
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * and results as sb_sym_eig, same kernels; the workspace is a device array inside the library
 * (about 2 MiB per GPU, held until the process ends), so the order is limited to
 * n <= SB_SYM_EIG_STATIC_MAX_N (-2 beyond).  The call allocates and frees nothing.  Every call on
 * one GPU uses that GPU's array: calls that overlap in time on one GPU (two streams, two threads)
 * race and must be serialised by the caller; calls on one stream are ordered by the stream.
 * Argument numbers: dt=1 n=2 S=3 V=4 lambda=5 sweeps=6 stream=7.
 */
#define SB_SYM_EIG_STATIC_MAX_N 256
int sb_sym_eig_static(sb_dtype dt, int64_t n, void *S, void *V, void *lambda, int sweeps, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SBTUCKER_H */
