"""CPU oracle for the Tucker decomposition by higher-order orthogonal iteration (Algorithm 1,
section II-C) and for the symmetric eigenproblem the GPU path uses inside it.

TEST INFRASTRUCTURE ONLY: imported by tests/ and the benchmark's cpu_baseline leg, never by the
product package.  Everything is numpy in fp64.  The steps are those of Algorithm 1 in its order
and notation; "leading left singular vectors" is numpy's SVD of the mode-r unfolding, the
contractions are written as the defining sums (einsum).  Nothing is shared with the GPU library,
which takes another route to the same subspaces (Gram matrix of the short side, Jacobi rotations).

Uniqueness: singular vectors are fixed up to sign (and up to a rotation inside a cluster of equal
singular values), so comparisons use what is unique: the projectors A A^T, B B^T, C C^T, the
reconstruction G x1 A x2 B x3 C, and the norm of the core.
"""
import numpy as np


def unfold(T, mode):
    """Mode-r unfolding T_(r) (Kolda & Bader): rows = mode r, columns = the other modes with the
    earlier mode running fastest."""
    return np.reshape(np.moveaxis(T, mode, 0), (T.shape[mode], -1), order="F")


def leading_left_singular_vectors(Y, r):
    """The r leading left singular vectors of the matrix Y as columns."""
    U, _, _ = np.linalg.svd(np.asarray(Y, dtype=np.float64), full_matrices=False)
    return U[:, :r]


def hosvd_init(T, core):
    """Step 2 of Algorithm 1: factor r <- leading left singular vectors of T_(r)."""
    return tuple(leading_left_singular_vectors(unfold(T, r), core[r]) for r in range(3))


def hooi(T, core, iterations, init=None):
    """Algorithm 1 for a third-order tensor T (m x n x p), core size (i, j, k).
    Returns A (m x i), B (n x j), C (p x k), G (i x j x k)."""
    T = np.asarray(T, dtype=np.float64)
    i, j, k = core
    A, B, C = hosvd_init(T, core) if init is None else (np.array(x, dtype=np.float64) for x in init)
    for _ in range(iterations):
        Y = np.einsum("mnp,nj,pk->mjk", T, B, C)                     # step 4
        A = leading_left_singular_vectors(unfold(Y, 0), i)           # step 5
        Y = np.einsum("mnp,mi,pk->ink", T, A, C)                     # step 6
        B = leading_left_singular_vectors(unfold(Y, 1), j)           # step 7
        Y = np.einsum("mnp,nj,mi->ijp", T, B, A)                     # step 8
        C = leading_left_singular_vectors(unfold(Y, 2), k)           # step 9
    G = np.einsum("mnp,mi,nj,pk->ijk", T, A, B, C)                   # step 11
    return A, B, C, G


def reconstruct(G, A, B, C):
    """T_mnp = G_ijk A_mi B_nj C_pk (section II-C)."""
    return np.einsum("ijk,mi,nj,pk->mnp", G, A, B, C)


def sym_eig(S):
    """Eigenvalues (descending) and eigenvectors (columns) of a real symmetric matrix."""
    w, V = np.linalg.eigh(np.asarray(S, dtype=np.float64))
    order = np.argsort(-w, kind="stable")
    return w[order], V[:, order]


def projector(U):
    return U @ U.T
