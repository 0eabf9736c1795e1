"""Pins of the CPU oracle against facts that do not come from the oracle itself.

The oracle evaluates eq. (1) (section II-B) and Listing 1 (section III-D).  Each test here fixes
it to something independent: hand-worked numbers, closed forms, pure mode permutations,
linearity, numpy's einsum / transpose-reshape-matmul (the conventional matricised evaluation of
section II-D), special cases that are textbook GEMM / GEMV / outer products, and the BLAS calls
printed in Table I.  Extents are pairwise different wherever possible so that any mix-up of two
indices or strides changes the answer.
"""
import itertools

import numpy as np
import pytest

from conftest import golden_lines
from oracle import oracle

EXT = dict(m=3, n=5, p=7, k=4, q=2)


def rand(shape, seed):
    return np.random.default_rng(seed).uniform(-1, 1, size=shape)


def all_cases_2x3():
    """(modesA, modesB) of the 36 order-2 x order-3 single-mode contractions into C_mnp."""
    out = []
    for free_a in "mnp":
        rest = [c for c in "mnp" if c != free_a]
        for ma in (free_a + "k", "k" + free_a):
            for perm in itertools.permutations(["k"] + rest):
                out.append((ma, "".join(perm)))
    return out


def test_case_enumeration_count():
    # section III-F: (|A|+|B|-2)! * |A| * |B| unique single-mode contractions; 36 for orders 2, 3
    cases = all_cases_2x3()
    assert len(cases) == len(set(cases)) == 36


def test_hand_worked_2x2x2():
    vals = {}
    for ln in golden_lines("hand_2x2x2.txt"):
        key, rest = ln.split(":")
        vals[key.strip()] = np.array([float(x) for x in rest.split()])
    A = vals["A"].reshape((2, 2), order="F")
    B = vals["B"].reshape((2, 2, 2), order="F")
    for wide in (True, False):
        C = oracle.contract("mk", A, "knp", B, "mnp", wide=wide)
        assert np.array_equal(C.ravel(order="F"), vals["C_alpha1_beta0"])
        C2 = oracle.contract("mk", A, "knp", B, "mnp", C=np.ones((2, 2, 2)), alpha=2.0, beta=-1.0, wide=wide)
        assert np.array_equal(C2.ravel(order="F"), vals["C_alpha2_betam1"])


@pytest.mark.parametrize("ma,mb", all_cases_2x3())
def test_identity_is_pure_permutation(ma, mb):
    # A = identity (free extent == K): C is B with its k mode renamed, permuted to (m,n,p): bitwise
    free_a = [c for c in ma if c != "k"][0]
    ext = dict(EXT)
    ext["k"] = ext[free_a]
    A = np.eye(ext["k"])
    B = rand([ext[c] for c in mb], 11)
    C = oracle.contract(ma, A, mb, B, "mnp")
    renamed = mb.replace("k", free_a)
    expect = np.transpose(B, [renamed.index(c) for c in "mnp"])
    assert np.array_equal(C, expect)


@pytest.mark.parametrize("ma,mb", all_cases_2x3())
def test_index_coded_closed_forms(ma, mb):
    # A == 1 and B depending only on its free indices  =>  C = K * B_free ; B == k => C = K(K-1)/2
    free_a = [c for c in ma if c != "k"][0]
    fb = [c for c in "mnp" if c != free_a]
    A = np.ones([EXT[c] for c in ma])
    grids = np.meshgrid(*[np.arange(EXT[c]) for c in mb], indexing="ij")
    g = dict(zip(mb, grids))
    B = (g[fb[0]] + 100.0 * g[fb[1]]).astype(np.float64)
    C = oracle.contract(ma, A, mb, B, "mnp")
    cg = dict(zip("mnp", np.meshgrid(*[np.arange(EXT[c]) for c in "mnp"], indexing="ij")))
    assert np.array_equal(C, EXT["k"] * (cg[fb[0]] + 100.0 * cg[fb[1]]))
    Bk = g["k"].astype(np.float64)
    Ck = oracle.contract(ma, A, mb, Bk, "mnp")
    assert np.array_equal(Ck, np.full(Ck.shape, EXT["k"] * (EXT["k"] - 1) / 2))
    # weights on A's free index as well: A = 1 + free_a, B = k  =>  C = (1 + free_a) K(K-1)/2
    ga = dict(zip(ma, np.meshgrid(*[np.arange(EXT[c]) for c in ma], indexing="ij")))
    Cw = oracle.contract(ma, 1.0 + ga[free_a], mb, Bk, "mnp")
    assert np.array_equal(Cw, (1.0 + cg[free_a]) * EXT["k"] * (EXT["k"] - 1) / 2)


@pytest.mark.parametrize("ma,mb", all_cases_2x3())
@pytest.mark.parametrize("wide", [True, False])
def test_matches_einsum_and_matricised_gemm(ma, mb, wide):
    A = rand([EXT[c] for c in ma], 1)
    B = rand([EXT[c] for c in mb], 2)
    C0 = rand([EXT[c] for c in "mnp"], 3)
    C = oracle.contract(ma, A, mb, B, "mnp", C=C0, alpha=0.75, beta=-0.5, wide=wide)
    ref = 0.75 * np.einsum("%s,%s->mnp" % (ma, mb), A, B) - 0.5 * C0
    assert np.allclose(C, ref, rtol=0, atol=1e-13)
    # conventional evaluation (section II-D): permute to C_IJ = A_IK B_KJ, one GEMM, permute back
    free_a = [c for c in ma if c != "k"][0]
    J = [c for c in mb if c != "k"]
    A_ik = np.transpose(A, [ma.index(free_a), ma.index("k")])
    B_kj = np.transpose(B, [mb.index("k")] + [mb.index(c) for c in J]).reshape(EXT["k"], -1)
    C_ij = (A_ik @ B_kj).reshape([EXT[free_a]] + [EXT[c] for c in J])
    order = [free_a] + J
    ref2 = 0.75 * np.transpose(C_ij, [order.index(c) for c in "mnp"]) - 0.5 * C0
    assert np.allclose(C, ref2, rtol=0, atol=1e-13)


def test_linearity_and_alpha_beta():
    A1, A2 = rand((3, 4), 5), rand((3, 4), 6)
    B = rand((5, 4, 7), 7)                                   # B_nkp
    C0 = rand((3, 5, 7), 8)
    f = lambda A, **kw: oracle.contract("mk", A, "nkp", B, "mnp", **kw)
    lhs = f(2.5 * A1 + A2)
    assert np.allclose(lhs, 2.5 * f(A1) + f(A2), rtol=0, atol=1e-13)
    ab = f(A1, C=C0, alpha=-1.25, beta=0.5)
    assert np.allclose(ab, -1.25 * f(A1) + 0.5 * C0, rtol=0, atol=1e-13)
    # swapping the roles of the two factors changes nothing
    sw = oracle.contract("nkp", B, "mk", A1, "mnp")
    assert np.array_equal(sw, f(A1))


def test_beta_zero_does_not_read_c():
    A, B = rand((3, 4), 1), rand((4, 5, 7), 2)
    Cnan = np.full((3, 5, 7), np.nan)
    C = oracle.contract("mk", A, "knp", B, "mnp", C=Cnan, alpha=1.0, beta=0.0)
    assert np.isfinite(C).all()
    Cflat = oracle.sb_gemm("N", "N", 3, 5, 4, 1.0, A.ravel(order="F"), 3, 0, B.ravel(order="F"), 4, 20,
                           0.0, Cnan.ravel(order="F"), 3, 15, 7)
    assert np.array_equal(Cflat.reshape((3, 5, 7), order="F"), C)


def test_order3_times_order3_two_batch_modes():
    # C_mpnq = A_mpk B_knq (the nested-batching example family of section III-F)
    A = rand((3, 7, 4), 21)
    B = rand((4, 5, 2), 22)
    C = oracle.contract("mpk", A, "knq", B, "mpnq")
    assert np.allclose(C, np.einsum("mpk,knq->mpnq", A, B), rtol=0, atol=1e-13)
    # Listing 2's example C_mn[p][q] = A_mk[p] B_nk[q]
    A2, B2 = rand((3, 4, 7), 23), rand((5, 4, 2), 24)
    C2 = oracle.contract("mkp", A2, "nkq", B2, "mnpq")
    assert np.allclose(C2, np.einsum("mkp,nkq->mnpq", A2, B2), rtol=0, atol=1e-13)


def test_general_contraction_more_than_one_summed_index():
    # eq. (1) allows any number of contracted indices; the matrix product of unfoldings pins it
    A, B = rand((3, 4, 6), 31), rand((6, 5, 4), 32)         # A_mkl  B_lnk
    C = oracle.contract("mkl", A, "lnk", B, "mn")
    ref = A.reshape(3, 24) @ np.transpose(B, (2, 0, 1)).reshape(24, 5)
    assert np.allclose(C, ref, rtol=0, atol=1e-13)
    # outer product (no contracted index: the GER case of section II-D)
    u, v = rand((3,), 33), rand((5,), 34)
    assert np.array_equal(oracle.contract("m", u, "n", v, "mn"), np.outer(u, v))
    # full contraction to a scalar-like order-0 result is a dot product
    w = rand((3,), 35)
    assert np.allclose(oracle.contract("m", u, "m", w, ""), np.dot(u, w), rtol=0, atol=1e-14)


def test_sampled_equals_full():
    A, B = rand((4, 3), 41), rand((7, 4, 5), 42)            # A_km B_pkn  (case 2.4)
    C0 = rand((3, 5, 7), 43)
    full = oracle.contract("km", A, "pkn", B, "mnp", C=C0, alpha=1.5, beta=2.0)
    idx = [(i, j, l) for i in range(3) for j in range(5) for l in range(7)]
    got = oracle.contract_at("km", A, "pkn", B, "mnp", idx, C=C0, alpha=1.5, beta=2.0)
    assert np.array_equal(got, np.array([full[t] for t in idx]))


def test_rejects_malformed_contractions():
    A, B = rand((3, 4), 1), rand((4, 5, 7), 2)
    # any order of the free indices in C is legal
    assert np.allclose(oracle.contract("mk", A, "knp", B, "pmn"), np.einsum("mk,knp->pmn", A, B), rtol=0, atol=1e-14)
    with pytest.raises(ValueError):
        oracle.contract("mk", A, "knp", B, "mnk")           # contracted index must not appear in C
    with pytest.raises(ValueError):
        oracle.contract("mk", A, "knp", B, "mn")            # free index missing from C
    with pytest.raises(ValueError):
        oracle.contract("mm", rand((3, 3), 1), "mnp", rand((3, 5, 7), 2), "np")   # repeated index
    with pytest.raises(ValueError):
        oracle.contract("mk", A, "knp", rand((5, 5, 7), 2), "mnp")               # k has two extents


# ---------------------------------------------------------------- Listing 1 (StridedBatchedGemm)

@pytest.mark.parametrize("opA,opB", [("N", "N"), ("N", "T"), ("T", "N"), ("T", "T")])
def test_sb_gemm_is_a_loop_of_textbook_gemms(opA, opB):
    m, n, k, batch = 3, 5, 4, 6
    lda, ldb, ldc = 9, 8, 7                                  # padded leading dimensions
    loa, lob, loc = 50, 45, 40
    a = rand((batch * loa + 100,), 51)
    b = rand((batch * lob + 100,), 52)
    c0 = rand((batch * loc + 100,), 53)
    c = oracle.sb_gemm(opA, opB, m, n, k, 1.5, a, lda, loa, b, ldb, lob, -0.5, c0, ldc, loc, batch)
    expect = c0.copy()
    for p in range(batch):
        ar, ac = (m, k) if opA == "N" else (k, m)
        br, bc = (k, n) if opB == "N" else (n, k)
        Ap = np.lib.stride_tricks.as_strided(a[p * loa:], (ar, ac), (8, 8 * lda))
        Bp = np.lib.stride_tricks.as_strided(b[p * lob:], (br, bc), (8, 8 * ldb))
        Ap = Ap if opA == "N" else Ap.T
        Bp = Bp if opB == "N" else Bp.T
        Cp = np.lib.stride_tricks.as_strided(expect[p * loc:], (m, n), (8, 8 * ldc))
        Cp[...] = 1.5 * (Ap @ Bp) - 0.5 * Cp
    assert np.allclose(c, expect, rtol=0, atol=1e-13)
    # nothing outside the m x n windows of C is touched
    mask = np.ones(c0.size, bool)
    for p in range(batch):
        for j in range(n):
            mask[p * loc + j * ldc: p * loc + j * ldc + m] = False
    assert np.array_equal(c[mask], c0[mask])


def test_sb_gemm_special_cases():
    a, b = rand((3, 4), 61), rand((4, 5), 62)
    af, bf = a.ravel(order="F"), b.ravel(order="F")
    # batch = 1: a plain GEMM
    c = oracle.sb_gemm("N", "N", 3, 5, 4, 1.0, af, 3, 0, bf, 4, 0, 0.0, np.zeros(15), 3, 0, 1)
    assert np.allclose(c.reshape((3, 5), order="F"), a @ b, rtol=0, atol=1e-14)
    # n = 1: a matrix-vector product
    c = oracle.sb_gemm("N", "N", 3, 1, 4, 1.0, af, 3, 0, bf, 4, 0, 0.0, np.zeros(3), 3, 0, 1)
    assert np.allclose(c, a @ b[:, 0], rtol=0, atol=1e-14)
    # k = 1: an outer product
    c = oracle.sb_gemm("N", "T", 3, 5, 1, 1.0, af, 3, 0, bf[:5], 5, 0, 0.0, np.zeros(15), 3, 0, 1)
    assert np.array_equal(c.reshape((3, 5), order="F"), np.outer(af[:3], bf[:5]))
    # stride 0 on the shared operand, interleaved batches in C (batch stride smaller than ldc)
    B3 = rand((4, 5, 7), 63)                                 # B_knp, batch over n, columns p
    c = oracle.sb_gemm("N", "N", 3, 7, 4, 1.0, af, 3, 0, B3.ravel(order="F"), 20, 4,
                       0.0, np.zeros(3 * 5 * 7), 15, 3, 5)
    assert np.allclose(c.reshape((3, 5, 7), order="F"), np.einsum("mk,knp->mnp", a, B3), rtol=0, atol=1e-14)


def _parse_ld(tok, ld):
    """'lda<1>' style token -> number, using the packed strides in `ld` (dict tensor -> list)."""
    if tok == "-":
        return 0
    if tok.isdigit():
        return int(tok)
    return ld[tok[2].upper()][int(tok[4])]


def test_table1_calls_reproduce_the_contraction():
    # Execute the calls printed in Table I with the oracle's GEMM and compare with eq. (1)
    # evaluated directly: pins the meaning of pointer offsets, ld and op in Listing 1.
    ext = dict(EXT)
    for ln in golden_lines("table1_blas_calls.txt"):
        f = [x.strip() for x in ln.split("|")]
        notation, loop, routine = f[0], f[1], f[2]
        ops = f[3].split()
        dims = f[4].split()
        lhs, rhs = notation.split("=")
        strip = lambda s: "".join(ch for ch in s.split("_")[1].replace("^T", "") if ch.isalpha())
        terms = rhs.split()
        modes = {t[0]: strip(t) for t in terms}
        modes["C"] = strip(lhs.strip())
        tens = {name: rand([ext[c] for c in modes[name]], 70 + i) for i, name in enumerate("AB")}
        ld = {name: oracle.packed_ld([ext[c] for c in modes[name]]) for name in "ABC"}
        size = lambda tok: int(np.prod([ext[c] for c in tok])) if tok != "-" else 1
        M, N, K = size(dims[0]), size(dims[1]), size(dims[2])
        first, second, cf = f[5].split(), f[6].split(), f[7].split()
        nloop = ext[loop] if loop != "-" else 1
        cbuf = np.zeros(int(np.prod([ext[c] for c in modes["C"]])))
        X, Y = tens[first[0]].ravel(order="F"), tens[second[0]].ravel(order="F")
        if routine == "GEMM":
            cbuf = oracle.sb_gemm(ops[0], ops[1], M, N, K, 1.0,
                                  X, _parse_ld(first[2], ld), _parse_ld(first[1], ld),
                                  Y, _parse_ld(second[2], ld), _parse_ld(second[1], ld),
                                  0.0, cbuf, _parse_ld(cf[1], ld), _parse_ld(cf[0], ld), nloop)
        else:
            # GEMV y = op(X) x with increments: a GEMM with one column per loop step whose
            # vector operand and result are read with the printed increments
            assert _parse_ld(second[2], ld) == 1             # incx = 1: x is a stored column
            incy = _parse_ld(cf[1], ld)
            for it in range(nloop):
                x0 = it * _parse_ld(second[1], ld)
                y = oracle.sb_gemm(ops[0], "N", M, 1, N, 1.0, X, _parse_ld(first[2], ld), 0,
                                   Y[x0:], N, 0, 0.0, np.zeros(M), M, 0, 1)
                cbuf[it * _parse_ld(cf[0], ld)::incy][:M] = y
        direct = oracle.contract(modes["A"], tens["A"], modes["B"], tens["B"], modes["C"])
        assert np.allclose(cbuf, direct.ravel(order="F"), rtol=0, atol=1e-13), notation


def test_wide_accumulation_is_more_accurate_than_the_fp64_gate():
    # a long sum with cancellation, against numpy's extended-precision sum of the same products
    K = 4096
    a = rand((1, K), 81)
    b = rand((K, 1, 1), 82)
    ref = np.sum(a[0].astype(np.longdouble) * b[:, 0, 0].astype(np.longdouble))
    scale = np.sum(np.abs(a[0] * b[:, 0, 0]))
    wide = oracle.contract("mk", a, "knp", b, "mnp", wide=True)[0, 0, 0]
    narrow = oracle.contract("mk", a, "knp", b, "mnp", wide=False)[0, 0, 0]
    assert abs(wide - float(ref)) <= 2e-16 * scale          # one final rounding to fp64
    assert abs(narrow - float(ref)) <= K * 1.2e-16 * scale
