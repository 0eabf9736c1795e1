"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Every comparison has two gates (helpers.assert_close): the relative Frobenius error within
1e-12 (fp64), 1e-5 (fp32), 2e-2 (bf16 in / fp32 accumulate / bf16 out), and every single element
within the running-error bound of the arithmetic, so that a few wrong elements cannot hide in a
norm over millions.  Elements of C outside the result windows must keep their bits.

A test that pins a kernel family never skips: FAMILY_TAKES states, from the contract in sbgemm.h,
which problems each family runs, the parameter lists are generated from it, and the family of the
launch is asserted."""
import itertools

import numpy as np
import pytest

import paper_1606_05696_amd as sb
from helpers import (TOL, assert_close, cases_2x3, from_dev, gemm_window_mask, packed, quantise, rel_fro,
                     strip_annotations, to_dev)
from oracle import oracle
from paper_1606_05696_amd import inputs

pytestmark = pytest.mark.gpu

KERNELS = {"auto": sb.SB_KERNEL_AUTO, "generic": sb.SB_KERNEL_GENERIC, "tiny": sb.SB_KERNEL_TINY, "mfma": sb.SB_KERNEL_MFMA,
           "thin": sb.SB_KERNEL_THIN, "panel": sb.SB_KERNEL_PANEL}


@pytest.fixture(autouse=True)
def _reset_kernel_choice():
    yield
    sb.sb_force_kernel(sb.SB_KERNEL_AUTO)


def sync():
    import torch
    torch.cuda.synchronize()


def family_takes(family, dtype, m, n, k):
    """Which N/T problems a kernel family runs when it is forced (sbgemm.h: sb_force_kernel)."""
    if family in ("auto", "generic"):
        return True
    if family == "thin":
        return 1 <= min(m, n) <= 4
    if family == "tiny":
        return dtype in ("f32", "f64") and m <= 32 and n <= 32 and k >= 1
    if family == "mfma":
        return k >= 1
    if family == "panel":
        return dtype == "bf16" and 1 <= k <= 128
    raise ValueError(family)


def run_sb_gemm(dtype, opA, opB, m, n, k, batch, lda, ldb, ldc, loa, lob, loc, alpha, beta, seed, kernel="auto", member=None):
    """One sb_gemm call on random buffers vs Listing 1 on the CPU, both gates plus untouched padding;
    a forced family must be the one that ran.  Returns (relative error, got, ref)."""
    assert family_takes(kernel, dtype, m, n, k), "the test's own table generated a problem this family does not take"
    rng = np.random.default_rng(seed)

    def span(op, rows, cols, ld, lo):
        r, c = (rows, cols) if op == "N" else (cols, rows)
        return max(1, (batch - 1) * lo + (c - 1) * ld + r + 3)

    a = quantise(rng.uniform(-1, 1, span(opA, m, k, lda, loa)), dtype)
    b = quantise(rng.uniform(-1, 1, span(opB, k, n, ldb, lob)), dtype)
    c0 = quantise(rng.uniform(-1, 1, span("N", m, n, ldc, loc)), dtype)
    dA, dB, dC = to_dev(a, dtype), to_dev(b, dtype), to_dev(c0, dtype)
    sb.sb_force_kernel(KERNELS[kernel])
    sb.sb_gemm(opA, opB, m, n, k, alpha, dA, lda, loa, dB, ldb, lob, beta, dC, ldc, loc, batch, dt=dtype)
    sync()
    if kernel != "auto":
        assert sb.sb_last_kernel() == KERNELS[kernel], (kernel, sb.sb_last_kernel(), dtype, opA, opB, m, n, k, batch)
    if member is not None:
        assert sb.sb_last_kernel_member() == member, (member, sb.sb_last_kernel_member(), dtype, opA, opB, m, n, k, batch, beta)
    ref = oracle.sb_gemm(opA, opB, m, n, k, alpha, a, lda, loa, b, ldb, lob, beta, c0, ldc, loc, batch,
                         wide=(dtype == "f64"))
    got = from_dev(dC)
    inside = gemm_window_mask(got.size, m, n, ldc, loc, batch)
    assert np.array_equal(got[~inside], c0[~inside]), "elements outside the m x n windows were written"
    err = assert_close(got[inside], ref[inside], dtype, k, np.abs(a).max(), np.abs(b).max(), alpha, beta, c0[inside],
                       what=(dtype, opA, opB, m, n, k, batch, kernel))
    return err, got, ref


RAGGED_CASES = [(dtype, kernel) for dtype in ("f64", "f32", "bf16") for kernel in ("auto", "generic", "mfma", "panel")
                if family_takes(kernel, dtype, 150, 77, 45)]
assert len(RAGGED_CASES) == 10


@pytest.mark.parametrize("dtype,kernel", RAGGED_CASES)
@pytest.mark.parametrize("opA,opB", [("N", "N"), ("N", "T"), ("T", "N"), ("T", "T")])
def test_sb_gemm_ragged_tiles(dtype, opA, opB, kernel):
    # several 64-wide tiles plus a ragged tail in every dimension, padded leading dimensions,
    # alpha and beta both active
    m, n, k, batch = 150, 77, 45, 3
    lda = (m if opA == "N" else k) + 3
    ldb = (k if opB == "N" else n) + 5
    ldc = m + 2
    loa = lda * (k if opA == "N" else m) + 7
    lob = ldb * (n if opB == "N" else k) + 1
    loc = ldc * n + 11
    err, got, ref = run_sb_gemm(dtype, opA, opB, m, n, k, batch, lda, ldb, ldc, loa, lob, loc, 0.75, -0.5, 7, kernel)
    assert err <= TOL[dtype], err


SHAPES = [(1, 1, 1, 1), (1, 9, 5, 4), (9, 1, 5, 4), (16, 16, 16, 1000), (8, 8, 8, 70001), (33, 17, 1, 3), (5, 6, 7, 2),
          (64, 64, 64, 5), (128, 128, 96, 2), (200, 130, 260, 2)]
# every (family, element type, shape) the family takes: 30 x auto, 30 x generic, 30 x mfma, 12 x tiny, 9 x thin, 9 x panel
SHAPE_CASES = [(dtype, kernel, m, n, k, batch) for dtype in ("f64", "f32", "bf16")
               for kernel in ("auto", "generic", "tiny", "mfma", "thin", "panel") for (m, n, k, batch) in SHAPES
               if family_takes(kernel, dtype, m, n, k)]
assert len(SHAPE_CASES) == 120


@pytest.mark.parametrize("dtype,kernel,m,n,k,batch", SHAPE_CASES)
def test_sb_gemm_shapes(dtype, kernel, m, n, k, batch):
    # stride 0 on A (shared operand, as in every order-2 x order-3 evaluation), packed B and C
    err, got, ref = run_sb_gemm(dtype, "N", "N", m, n, k, batch, m, k, m, 0, k * n, m * n, 1.0, 0.0, 11, kernel)
    assert err <= TOL[dtype], err
    err, got, ref = run_sb_gemm(dtype, "T", "N", m, n, k, batch, k, k, m, m * k, 0, m * n, -1.5, 1.0, 12, kernel)
    assert err <= TOL[dtype], err


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("opA,opB", [("N", "N"), ("N", "T"), ("T", "N"), ("T", "T")])
def test_sb_gemm_tiny_short_batches_of_32(dtype, opA, opB):
    # the tiny-matrix kernel runs a SHORT batch of 32-wide problems as independent 16 x 16 blocks (extra
    # batch digits: row half, column half): split in both, in m only, in n only; k below, at and beyond one
    # step of 16; batch 1, odd and the largest that is still split; padded leading dimensions; a shared
    # operand; alpha and beta.  The last two shapes are not split (300 problems; m not 32) and run as before.
    for m, n, k, batch, pad, share in ((32, 32, 32, 32, 0, ""), (32, 32, 7, 1, 1, ""), (32, 16, 40, 9, 1, "A"), (8, 32, 16, 33, 1, "B"),
                                       (32, 32, 64, 256, 0, ""), (32, 32, 5, 300, 1, ""), (24, 32, 20, 6, 1, "")):
        split = batch <= 256 and m in (32, 8) and (m, n) != (24, 32)
        lda = (m if opA == "N" else k) + 3 * pad
        ldb = (k if opB == "N" else n) + 5 * pad
        ldc = m + 2 * pad
        loa = 0 if share == "A" else lda * (k if opA == "N" else m) + 7 * pad
        lob = 0 if share == "B" else ldb * (n if opB == "N" else k) + pad
        loc = ldc * n + 11 * pad
        for alpha, beta in ((1.0, 0.0), (0.75, -0.5)):
            run_sb_gemm(dtype, opA, opB, m, n, k, batch, lda, ldb, ldc, loa, lob, loc, alpha, beta, seed=m + n + k + batch,
                        kernel="tiny", member=sb.SB_MEMBER_TINY_BLOCKS if split else sb.SB_MEMBER_TINY_WHOLE)


def test_tiny_short_batches_of_32_in_a_nest():
    # the split adds its digits on top of a nest that already has more than two levels
    for dtype in ("f64", "f32"):
        err, text = contract_case(dtype, "mk", "kn[p][q][r]", "mn[p][q][r]", dict(m=32, n=32, k=24, p=3, q=2, r=5), seed=17,
                                  kernel="tiny", alpha=0.5, beta=2.0)
        assert err <= TOL[dtype], (text, err)


@pytest.mark.parametrize("dtype", ["f64", "f32", "bf16"])
@pytest.mark.parametrize("opA,opB", [("N", "N"), ("N", "T"), ("T", "N"), ("T", "T")])
@pytest.mark.parametrize("thin", [1, 2, 3, 4])
def test_sb_gemm_thin_shapes(dtype, opA, opB, thin):
    # the BatchedGemv end: n (then m) is the thin extent, the other two are several tiles with ragged
    # tails.  Packed and whole-vector extents take the 16-byte kernels, the padded odd ones the scalar
    # kernels; a long k exercises the unrolled trips and their tail; the last two have enough rows
    # for the widest loads, with sixteen and with four waves to a workgroup.
    for m, n, k, batch, pad in [(1000, thin, 333, 3, 1), (thin, 1000, 333, 3, 1), (1024, thin, 520, 5, 0),
                                (thin, 1024, 520, 5, 0), (8, thin, 4099, 2, 0), (thin, 24, 8192, 4, 0),
                                (4096, thin, 136, 16, 0), (4096, thin, 96, 70, 0)]:
        lda = (m if opA == "N" else k) + 3 * pad
        ldb = (k if opB == "N" else n) + 5 * pad
        ldc = m + 2 * pad
        loa = lda * (k if opA == "N" else m) + 7 * pad
        lob = ldb * (n if opB == "N" else k) + pad
        loc = ldc * n + 11 * pad
        err, got, ref = run_sb_gemm(dtype, opA, opB, m, n, k, batch, lda, ldb, ldc, loa, lob, loc, 0.75, -0.5, 21,
                                    "thin")
        assert sb.sb_last_kernel() == sb.SB_KERNEL_THIN
        assert err <= TOL[dtype], (m, n, k, err)
        err, got, ref = run_sb_gemm(dtype, opA, opB, m, n, k, batch, lda, ldb, ldc, loa, lob, loc, 1.0, 0.0, 22)
        assert err <= TOL[dtype], (m, n, k, err)


@pytest.mark.parametrize("dtype", ["f64", "f32", "bf16"])
def test_thin_blas_conventions(dtype):
    # thin shapes with alpha == 0 (operands full of NaN are not read), k == 0, and beta == 0 over a C
    # full of NaN (not read either)
    m, n, k, batch = 300, 2, 40, 3
    rng = np.random.default_rng(9)
    a = quantise(rng.uniform(-1, 1, m * k * batch), dtype)
    b = quantise(rng.uniform(-1, 1, k * n), dtype)
    c0 = quantise(rng.uniform(-1, 1, m * n * batch), dtype)
    dA, dB = to_dev(a, dtype), to_dev(b, dtype)
    dNaN = to_dev(np.full(m * k * batch, np.nan), dtype)
    dC = to_dev(c0, dtype)
    sb.sb_gemm("N", "N", m, n, k, 0.0, dNaN, m, m * k, dNaN, k, 0, 0.5, dC, m, m * n, batch, dt=dtype)
    assert sb.sb_last_kernel() == sb.SB_KERNEL_THIN
    assert_close(from_dev(dC), 0.5 * c0, dtype, 0, 1.0, 1.0, 0.0, 0.5, c0)
    dC = to_dev(c0, dtype)
    sb.sb_gemm("N", "N", m, n, 0, 1.0, dA, m, 0, dB, 1, 0, 0.0, dC, m, m * n, batch, dt=dtype)
    assert np.array_equal(from_dev(dC), np.zeros(m * n * batch))
    dC = to_dev(np.full(m * n * batch, np.nan), dtype)
    sb.sb_gemm("N", "N", m, n, k, 1.0, dA, m, m * k, dB, k, 0, 0.0, dC, m, m * n, batch, dt=dtype)
    ref = oracle.sb_gemm("N", "N", m, n, k, 1.0, a, m, m * k, b, k, 0, 0.0, np.zeros_like(c0), m, m * n, batch)
    assert_close(from_dev(dC), ref, dtype, k, 1.0, 1.0)
    sync()


def test_thin_calls_take_the_thin_kernels():
    # a batched matrix-vector product and a batched vector-matrix product, many 16-byte tiles: the
    # selector sends both to the level-2 family, shared operand (stride 0) included
    for m, n in [(4096, 1), (1, 4096), (2048, 3), (2, 2048)]:
        err, got, ref = run_sb_gemm("f32", "N", "N", m, n, 256, 40, m, 256, m, 0, 256 * n, m * n, 1.0, 0.0, 31)
        assert sb.sb_last_kernel() == sb.SB_KERNEL_THIN
        assert err <= TOL["f32"], err
        err, got, ref = run_sb_gemm("f64", "T", "T", m, n, 256, 40, 256, n, m, m * 256, 0, m * n, 1.0, 0.0, 32)
        assert sb.sb_last_kernel() == sb.SB_KERNEL_THIN
        assert err <= TOL["f64"], err


@pytest.mark.parametrize("dtype", ["f64", "f32", "bf16"])
def test_blas_conventions(dtype):
    import torch
    m, n, k, batch = 20, 10, 8, 3
    rng = np.random.default_rng(5)
    a = quantise(rng.uniform(-1, 1, m * k), dtype)
    b = quantise(rng.uniform(-1, 1, k * n * batch), dtype)
    c0 = quantise(rng.uniform(-1, 1, m * n * batch), dtype)
    dA, dB = to_dev(a, dtype), to_dev(b, dtype)
    # beta == 0: C is not read, NaNs in it vanish
    dC = to_dev(np.full(m * n * batch, np.nan), dtype)
    sb.sb_gemm("N", "N", m, n, k, 1.0, dA, m, 0, dB, k, k * n, 0.0, dC, m, m * n, batch, dt=dtype)
    got = from_dev(dC)
    ref = oracle.sb_gemm("N", "N", m, n, k, 1.0, a, m, 0, b, k, k * n, 0.0, np.zeros_like(c0), m, m * n, batch)
    assert_close(got, ref, dtype, k, 1.0, 1.0)
    # alpha == 0: A and B are not read (NaNs in them are harmless), C = beta*C
    dAn = to_dev(np.full(m * k, np.nan), dtype)
    dC = to_dev(c0, dtype)
    sb.sb_gemm("N", "N", m, n, k, 0.0, dAn, m, 0, dB, k, k * n, 0.5, dC, m, m * n, batch, dt=dtype)
    assert_close(from_dev(dC), 0.5 * c0, dtype, 0, 1.0, 1.0, 0.0, 0.5, c0)
    # k == 0 with beta == 0 zeroes C
    dC = to_dev(c0, dtype)
    sb.sb_gemm("N", "N", m, n, 0, 1.0, dA, m, 0, dB, 1, 0, 0.0, dC, m, m * n, batch, dt=dtype)
    assert np.array_equal(from_dev(dC), np.zeros(m * n * batch))
    # empty problems touch nothing
    dC = to_dev(c0, dtype)
    sb.sb_gemm("N", "N", 0, n, k, 1.0, dA, 1, 0, dB, k, k * n, 0.0, dC, 1, m * n, batch, dt=dtype)
    sb.sb_gemm("N", "N", m, n, k, 1.0, dA, m, 0, dB, k, k * n, 0.0, dC, m, m * n, 0, dt=dtype)
    assert np.array_equal(from_dev(dC), quantise(c0, dtype))
    torch.cuda.synchronize()


def contract_case(dtype, ma, mb, mc, ext, strat="auto", alpha=1.0, beta=0.0, seed=0, pad=None, kernel="auto",
                  tensors=None):
    """sb_contract on device vs the oracle, both gates (Frobenius norm and element-wise bound) plus
    untouched padding; mode strings may be annotated.  Returns (error, plan text)."""
    pa, pb, pc = (strip_annotations(s) for s in (ma, mb, mc))
    dA, dB, dC = ([ext[c] for c in s] for s in (pa, pb, pc))
    if tensors is None:
        A = inputs.make_tensor(seed, dA, dtype)
        B = inputs.make_tensor(seed + 1, dB, dtype)
    else:
        A, B = tensors
    C0 = quantise(inputs.uniform_tensor(seed + 2, dC), dtype)
    sA = sB = sC = None
    hA, hB, hC = A, B, C0
    if pad:                       # embed each tensor in a larger packed one: padded strides
        def embed(X, extra):
            big = np.zeros([d + e for d, e in zip(X.shape, extra)], dtype=X.dtype, order="F")
            big[tuple(slice(0, d) for d in X.shape)] = X
            return big, packed(big.shape)
        hA, sA = embed(A, pad[0])
        hB, sB = embed(B, pad[1])
        hC, sC = embed(C0, pad[2])
    tA, tB, tC = to_dev(hA, dtype), to_dev(hB, dtype), to_dev(hC, dtype)
    sb.sb_force_kernel(KERNELS[kernel])
    rc, plan = sb.sb_contract_plan(ma, mb, mc, dA, dB, stridesA=sA, stridesB=sB, stridesC=sC, strat=strat)
    sb.sb_contract(ma, mb, mc, alpha, tA, dA, tB, dB, beta, tC, dC, stridesA=sA, stridesB=sB, stridesC=sC,
                   strat=strat, dt=dtype)
    sync()
    if kernel != "auto":
        assert sb.sb_last_kernel() == KERNELS[kernel], (kernel, sb.sb_last_kernel(), plan.text())
    ref = oracle.contract(pa, A, pb, B, pc, C=C0, alpha=alpha, beta=beta, wide=(dtype == "f64"))
    got = from_dev(tC, hC.shape)
    if pad:
        inner = tuple(slice(0, d) for d in C0.shape)
        outside = got.copy()
        outside[inner] = 0
        assert not outside.any(), "padding of C was written"
        got = got[inner]
    K = int(np.prod([ext[c] for c in set(pa) & set(pb)], dtype=np.int64))
    err = assert_close(got, ref, dtype, K, np.abs(A).max() if A.size else 0.0, np.abs(B).max() if B.size else 0.0,
                       alpha, beta, C0, what=(dtype, ma, mb, mc, strat, kernel, plan.text()))
    return err, plan.text()


def test_cfg1_small_reference_case():
    # C_mnp = A_mk B_knp, 32^4, fp64: strided-batched over p, plus the other two legal evaluations
    w = inputs.WORKLOADS[1]
    A, B = inputs.workload_tensors(1)
    for ma, mb, mc in (w["eval"], ("mk", "k[n]p", "m[n]p"), ("mk", "k(np)", "m(np)")):
        err, text = contract_case("f64", ma, mb, mc, w["ext"], tensors=(A, B))
        assert err <= TOL["f64"], (text, err)
        err, text = contract_case("f64", ma, mb, mc, w["ext"], alpha=0.75, beta=-0.5, tensors=(A, B))
        assert err <= TOL["f64"], (text, err)


@pytest.mark.parametrize("strat", ["auto", "flatten", "batch_last", "batch_mid", "level2"])
def test_cfg2_all_36_cases_at_64(strat):
    # every order-2 x order-3 contraction at dim 64, fp32, every strategy: the 8 flattened GEMMs,
    # the 32 StridedBatchedGemm evaluations, the extended-operation and matrix-vector forms
    ext = dict(m=64, n=64, p=64, k=64)
    done = 0
    for i, (ma, mb) in enumerate(cases_2x3()):
        rc, plan = sb.sb_contract_plan(ma, mb, "mnp", [64, 64], [64, 64, 64], strat=strat, check=False)
        if rc == sb.SB_ERR_ILLEGAL_EVAL:
            continue
        err, text = contract_case("f32", ma, mb, "mnp", ext, strat=strat, seed=20 + i)
        assert err <= TOL["f32"], (text, err)
        done += 1
    # 12 cases have no [p] form and 12 no [n] form even with an extended operation: the GEMM's
    # column mode would have to come from the tensor that already supplies the rows
    assert done == {"auto": 36, "flatten": 8, "batch_last": 24, "batch_mid": 24, "level2": 36}[strat]


@pytest.mark.parametrize("dtype", ["f64", "f32", "bf16"])
def test_all_36_cases_odd_extents_alpha_beta_padding(dtype):
    ext = dict(m=37, n=21, p=13, k=29)
    for i, (ma, mb) in enumerate(cases_2x3()):
        err, text = contract_case(dtype, ma, mb, "mnp", ext, alpha=0.75, beta=-0.5, seed=100 + i)
        assert err <= TOL[dtype], (text, err)
        pad = ([1, 0], [2, 0, 1], [3, 1, 0])
        err, text = contract_case(dtype, ma, mb, "mnp", ext, strat="nested", alpha=1.0, beta=0.0, seed=200 + i, pad=pad)
        assert err <= TOL[dtype], (text, err)


@pytest.mark.parametrize("kernel", ["auto", "generic", "tiny"])
def test_cfg3_tiny_batch_full_size(kernel):
    # m = n = k = 16, p = 65536, fp32: the bandwidth-bound regime, compared element by element
    w = inputs.WORKLOADS[3]
    A, B = inputs.workload_tensors(3)
    err, text = contract_case("f32", *w["eval"], w["ext"], tensors=(A, B), kernel=kernel)
    assert err <= TOL["f32"], (text, err)


def sample_indices(dimsC, n, seed):
    """Random output positions plus the corners and tile-boundary positions of every mode."""
    rng = np.random.default_rng(seed)
    idx = [tuple(int(rng.integers(0, d)) for d in dimsC) for _ in range(n)]
    edge = [sorted({0, 1, d // 2 - 1, d // 2, d - 2, d - 1} & set(range(d))) for d in dimsC]
    idx += list(itertools.islice(itertools.product(*edge), 4096))
    return np.array(sorted(set(idx)), dtype=np.int64)


@pytest.mark.parametrize("cfg", [40, 41])
@pytest.mark.parametrize("form", ["eval", "mid", "flat"])
def test_cfg4_large_cube_full_size_sampled(cfg, form):
    # C_mnp = A_km B_knp at 512^4 in the launch configuration the benchmark times; 68.7 G
    # multiply-adds are too many for the CPU loop, so a few thousand outputs are checked one by one
    w = inputs.WORKLOADS[cfg]
    dtype = w["dtype"]
    A, B = inputs.workload_tensors(cfg)
    ma, mb, mc = {"eval": w["eval"], "mid": ("km", "k[n]p", "m[n]p"), "flat": ("km", "k(np)", "m(np)")}[form]
    dA, dB, dC = ([w["ext"][c] for c in strip_annotations(s)] for s in (ma, mb, mc))
    tA, tB = to_dev(A, dtype), to_dev(B, dtype)
    tC = to_dev(np.full(1, np.nan), dtype).repeat(int(np.prod(dC)))
    sb.sb_contract(ma, mb, mc, 1.0, tA, dA, tB, dB, 0.0, tC, dC, dt=dtype)
    sync()
    got_full = from_dev(tC, dC)
    assert np.isfinite(got_full).all()
    idx = sample_indices(dC, 6000, 404)
    ref = oracle.contract_at("km", A, "knp", B, "mnp", idx, wide=(dtype == "f64"))
    got = got_full[idx[:, 0], idx[:, 1], idx[:, 2]]
    assert_close(got, ref, dtype, 512, 1.0, 1.0, what=(cfg, form))
    assert np.max(np.abs(got - ref)) <= 50 * TOL[dtype] * np.sqrt(512 / 3)       # no single wild element


def test_cfg4b_full_size_every_element():
    # the benchmark's headline launch, C_mnp = A_km B_knp at 512^4 in fp32 batched over p, compared
    # with the oracle in every one of its 134 million outputs (the oracle's plain loop takes a few
    # seconds on the test machine's cores)
    w = inputs.WORKLOADS[41]
    A, B = inputs.workload_tensors(41)
    ma, mb, mc = w["eval"]
    dA, dB, dC = ([w["ext"][c] for c in w[t]] for t in "ABC")
    tA, tB = to_dev(A, "f32"), to_dev(B, "f32")
    tC = to_dev(np.full(1, np.nan), "f32").repeat(int(np.prod(dC)))
    sb.sb_contract(ma, mb, mc, 1.0, tA, dA, tB, dB, 0.0, tC, dC, dt="f32")
    sync()
    assert sb.sb_last_kernel() == sb.SB_KERNEL_MFMA
    got = from_dev(tC, dC)
    del tC
    ref = oracle.contract("km", A, "knp", B, "mnp", wide=False)
    assert_close(got, ref, "f32", 512, 1.0, 1.0, what="cfg4b, every element")


def test_cfg4_shape_reduced_full_compare():
    for dtype in ("f64", "f32"):
        err, text = contract_case(dtype, "km", "kn[p]", "mn[p]", dict(m=192, n=160, p=5, k=136), seed=41)
        assert err <= TOL[dtype], (text, err)


def test_cfg5_order3_x_order3_full_size():
    # C_mpnq = A_mpk B_knq, 64^4 x 128, bf16 in / fp32 accumulate: nested batching over (p,q) in one
    # launch, the flattened GEMM and the two partly flattened forms, all against one oracle result
    w = inputs.WORKLOADS[5]
    A, B = inputs.workload_tensors(5)
    ref = oracle.contract("mpk", A, "knq", B, "mpnq", wide=False)
    dA, dB, dC = list(A.shape), list(B.shape), list(ref.shape)
    tA, tB = to_dev(A, "bf16"), to_dev(B, "bf16")
    forms = [w["eval"], ("(mp)k", "k(nq)", "(mp)(nq)"), ("(mp)k", "kn[q]", "(mp)n[q]"), ("m[p]k", "k(nq)", "m[p](nq)")]
    for ma, mb, mc in forms:
        tC = to_dev(np.full(1, np.nan), "bf16").repeat(ref.size)
        sb.sb_contract(ma, mb, mc, 1.0, tA, dA, tB, dB, 0.0, tC, dC, dt="bf16")
        sync()
        assert sb.sb_last_kernel() == sb.SB_KERNEL_PANEL and sb.sb_last_kernel_member() == sb.SB_MEMBER_PANEL_WIDE, mc
        assert_close(from_dev(tC, dC), ref, "bf16", 128, np.abs(A).max(), np.abs(B).max(), what=mc)
    # same contraction in fp32 and fp64 at reduced extents, with alpha and beta
    ext = dict(m=24, p=5, n=40, q=3, k=50)
    for dtype in ("f64", "f32", "bf16"):
        for strat in ("auto", "nested"):
            err, text = contract_case(dtype, "mpk", "knq", "mpnq", ext, strat=strat, alpha=-0.5, beta=2.0, seed=55)
            assert err <= TOL[dtype], (text, err)


@pytest.mark.parametrize("ma,mb,mc", [("m[p]k", "kn[q]", "m[p]n[q]"), ("k[p]m", "nk[q]", "m[p]n[q]"), ("mk[p]", "nk[q]", "mn[p][q]"),
                                      ("km[p]", "kn[q]", "mn[p][q]"), ("m[p]k", "kn[q]", "mn[p][q]")])
def test_two_level_batches_with_one_operand_per_level(ma, mb, mc):
    # C_..[p]..[q] = A_..[p] B_..[q]: every A_p meets every B_q (the nested example of section III-F);
    # ragged group counts, all operand orientations, short and full k, m and n below and at 64
    for ext in (dict(m=64, n=64, p=6, q=5, k=128), dict(m=40, n=24, p=9, q=4, k=72), dict(m=64, n=48, p=4, q=7, k=32),
                dict(m=36, n=24, p=5, q=6, k=40)):
        for dtype, kernel in (("bf16", "panel"), ("bf16", "mfma"), ("f32", "auto")):
            err, text = contract_case(dtype, ma, mb, mc, ext, seed=91, kernel=kernel)
            assert err <= TOL[dtype], (text, ext, err)
            err, text = contract_case(dtype, ma, mb, mc, ext, alpha=0.5, beta=-1.0, seed=92, kernel=kernel)
            assert err <= TOL[dtype], (text, ext, err)


@pytest.mark.parametrize("opA,opB", [("N", "N"), ("N", "T"), ("T", "N"), ("T", "T")])
def test_panel_grid_kernel(opA, opB):
    # the whole-k panel-grid kernel on plain (batched) GEMMs: several blocks of 4 x 4 panels with ragged
    # last panels and a ragged last block, extents that are and are not whole 16-byte vectors, odd leading
    # dimensions (vector accesses at 2-byte alignment), short and full k, a shared operand (the batch then
    # extends the other operand's side of the grid), beta = 0 and beta != 0
    for m, n, k, batch, pad, share in ((520, 328, 128, 2, 0, ""), (300, 200, 100, 3, 1, ""), (333, 270, 77, 2, 1, "A"),
                                       (64, 64, 128, 37, 0, "B"), (40, 24, 72, 23, 1, "A"), (256, 512, 16, 1, 0, ""),
                                       (257, 65, 8, 2, 1, ""), (7, 300, 3, 5, 1, "B")):
        lda = (m if opA == "N" else k) + 3 * pad
        ldb = (k if opB == "N" else n) + 5 * pad
        ldc = m + 1 * pad
        loa = 0 if share == "A" else lda * (k if opA == "N" else m) + 7 * pad
        lob = 0 if share == "B" else ldb * (n if opB == "N" else k) + pad
        loc = ldc * n + 11 * pad
        for alpha, beta in ((1.0, 0.0), (0.75, -0.5)):
            run_sb_gemm("bf16", opA, opB, m, n, k, batch, lda, ldb, ldc, loa, lob, loc, alpha, beta, seed=m + n + k,
                        kernel="panel")


@pytest.mark.parametrize("opA,opB", [("N", "N"), ("N", "T"), ("T", "N"), ("T", "T")])
def test_panel_grid_kernel_wide_blocks(opA, opB):
    # the member of the panel-grid kernel that loads straight into LDS (blocks of 2 x 8 panels): k = 128,
    # beta = 0, whole 64-wide panels in whole blocks, everything 16-byte aligned.  One and several blocks
    # along either side, padded leading dimensions, independent batches, a shared operand (the batch then
    # extends the other operand's side of the grid), alpha != 1.  beta != 0 runs the same shapes through the
    # 4 x 4 member.
    for m, n, batch, pad, share in ((128, 512, 1, 0, ""), (512, 1024, 1, 8, ""), (384, 512, 3, 16, ""), (64, 512, 6, 8, "B"),
                                    (128, 64, 8, 24, "A"), (640, 1536, 2, 0, "")):
        k = 128
        lda = (m if opA == "N" else k) + pad
        ldb = (k if opB == "N" else n) + 2 * pad
        ldc = m + pad
        loa = 0 if share == "A" else lda * (k if opA == "N" else m) + 8 * pad
        lob = 0 if share == "B" else ldb * (n if opB == "N" else k) + 16 * pad
        loc = ldc * n + 8 * pad
        for alpha, beta in ((1.0, 0.0), (-0.75, 0.0), (0.5, 1.5)):
            run_sb_gemm("bf16", opA, opB, m, n, k, batch, lda, ldb, ldc, loa, lob, loc, alpha, beta, seed=m + n + batch,
                        kernel="panel", member=sb.SB_MEMBER_PANEL_WIDE if beta == 0.0 else sb.SB_MEMBER_PANEL_4X4)
    # one element off 16-byte alignment, one odd leading dimension: the 4 x 4 member
    run_sb_gemm("bf16", opA, opB, 128, 512, 128, 1, 129 if opA == "N" else 128, 128 if opB == "N" else 512, 128, 0, 0, 0, 1.0, 0.0,
                seed=3, kernel="panel", member=sb.SB_MEMBER_PANEL_WIDE if opA == "T" else sb.SB_MEMBER_PANEL_4X4)


def test_panel_grid_kernel_wide_blocks_two_independent_levels():
    # sb_gemm2 with both levels moving both operands: two outer indices of independent panel grids; and with
    # level 0 moving A only and level 1 moving both (a row-side digit plus an outer index)
    m, n, k, b0, b1 = 128, 512, 128, 2, 3
    rng = np.random.default_rng(77)
    for share_b in (False, True):
        A = inputs.round_to_bf16(rng.standard_normal((b1, b0, k, m)).astype(np.float32)).astype(np.float64)       # [q][p][k][m]: column-major m x k
        B = inputs.round_to_bf16(rng.standard_normal((b1, 1 if share_b else b0, n, k)).astype(np.float32)).astype(np.float64)
        tA, tB = to_dev(A.reshape(-1), "bf16"), to_dev(B.reshape(-1), "bf16")
        tC = to_dev(np.zeros(b1 * b0 * n * m), "bf16")
        sb.sb_force_kernel(sb.SB_KERNEL_PANEL)
        sb.sb_gemm2("N", "N", m, n, k, 0.5, tA, m, k * m, b0 * k * m, tB, k, 0 if share_b else n * k, (1 if share_b else b0) * n * k,
                    0.0, tC, m, n * m, b0 * n * m, b0, b1, dt="bf16")
        sync()
        assert sb.sb_last_kernel() == sb.SB_KERNEL_PANEL and sb.sb_last_kernel_member() == sb.SB_MEMBER_PANEL_WIDE
        got = from_dev(tC).reshape(b1, b0, n, m)
        for q in range(b1):
            for p_ in range(b0):
                Ap = A[q, p_].T                                   # m x k (A[q][p] is k x m in C order, i.e. column-major m x k)
                Bp = B[q, 0 if share_b else p_].T                 # k x n
                ref = 0.5 * (Ap @ Bp)                             # m x n
                assert_close(got[q, p_].T, ref, "bf16", k, np.abs(A).max(), np.abs(B).max(), 0.5, what=(share_b, p_, q))
    sb.sb_force_kernel(sb.SB_KERNEL_AUTO)


@pytest.mark.parametrize("ma,mb,mc", [("m[p]k", "kn[q]", "m[p]n[q]"), ("k[p]m", "nk[q]", "m[p]n[q]"), ("mk[p]", "nk[q]", "mn[p][q]"),
                                      ("km[p]", "kn[q]", "mn[p][q]")])
def test_panel_grid_kernel_wide_blocks_nested(ma, mb, mc):
    # nests whose row side counts p and whose column side counts q in whole blocks of 2 x 8 panels, and
    # extents of 128 that put two panels of one matrix next to the batch digit on either side
    for ext in (dict(m=64, n=64, p=6, q=8, k=128), dict(m=128, n=64, p=3, q=16, k=128), dict(m=64, n=128, p=4, q=4, k=128)):
        for alpha in (1.0, 0.5):
            err, text = contract_case("bf16", ma, mb, mc, ext, alpha=alpha, seed=93, kernel="panel")
            assert err <= TOL["bf16"], (text, ext, err)
            assert sb.sb_last_kernel_member() == sb.SB_MEMBER_PANEL_WIDE, (text, ext)


def test_panel_grid_kernel_is_selected_for_the_large_short_k_products():
    # flat bf16 GEMMs with k <= 128 and at least 128 blocks of 256 x 256: the selector's own choice
    err, got, ref = run_sb_gemm("bf16", "N", "N", 4096, 2048, 64, 1, 4096, 64, 4096, 0, 0, 0, 1.0, 0.0, seed=5)
    assert sb.sb_last_kernel() == sb.SB_KERNEL_PANEL
    err, got, ref = run_sb_gemm("bf16", "T", "N", 1024, 1024, 128, 8, 128, 128, 1024, 128 * 1024, 128 * 1024, 1024 * 1024,
                                1.0, 0.0, seed=6)
    assert sb.sb_last_kernel() == sb.SB_KERNEL_PANEL


@pytest.mark.parametrize("kernel", ["auto", "generic", "mfma"])
def test_bf16_output_rounding_is_nearest_even(kernel):
    # k = 1 and B = 1: C = alpha * a, one fp32 multiply and one rounding; both sides round the same
    # fp32 number, so the bf16 bit patterns must agree exactly
    import torch
    m, n, batch = 96, 64, 70
    a = inputs.normal_bf16_tensor(7, [m * batch])
    a[:8] = [1.0, 1.00390625, 1.01171875, -1.00390625, 0.0, 3.0e38, -3.0e38, 1e-40]     # ties, overflow, denormal
    a = inputs.round_to_bf16(a)
    alpha = np.float32(1.0) / np.float32(3.0)
    tA, tB = to_dev(a, "bf16"), to_dev(np.ones(n), "bf16")
    tC = to_dev(np.zeros(m * n * batch), "bf16")
    sb.sb_force_kernel(KERNELS[kernel])
    sb.sb_gemm("N", "N", m, n, 1, float(alpha), tA, m, m, tB, 1, 0, 0.0, tC, m, m * n, batch, dt="bf16")
    sync()
    if kernel != "auto":
        assert sb.sb_last_kernel() == KERNELS[kernel]
    want = inputs.bf16_bits(inputs.round_to_bf16((a.astype(np.float32) * alpha).astype(np.float32)))
    got = tC.view(torch.int16).cpu().numpy().view(np.uint16).reshape(batch, n, m)
    assert np.array_equal(got, np.broadcast_to(want.reshape(batch, 1, m), got.shape))


def test_three_and_four_level_nests():
    # batch levels that nest in every tensor are merged into one launch; the others loop on the host
    ext = dict(m=20, n=12, p=3, q=4, r=2, s=3, k=9)
    for ma, mb, mc in (("mpk", "knqr", "mnpqr"), ("mpk", "knqr", "mnqpr"), ("mpk", "knqrs", "mnpqrs"), ("kpm", "qnkr", "mrnpq")):
        err, text = contract_case("f32", ma, mb, mc, ext, strat="nested", alpha=0.5, beta=-1.0, seed=77)
        assert err <= TOL["f32"], (text, err)


NESTED_CASES = [("f32", "generic", "N", "T", 37, 21, 13), ("f64", "tiny", "T", "N", 16, 9, 20), ("f32", "tiny", "N", "N", 32, 32, 8),
                ("f32", "mfma", "N", "N", 70, 40, 24), ("f64", "mfma", "T", "N", 128, 128, 64), ("f32", "mfma", "T", "N", 128, 256, 96),
                ("bf16", "mfma", "T", "N", 128, 128, 256), ("bf16", "mfma", "N", "T", 50, 90, 40), ("bf16", "generic", "N", "N", 20, 30, 10),
                ("f32", "auto", "N", "N", 3, 50, 64), ("bf16", "auto", "N", "N", 64, 64, 128)]


@pytest.mark.parametrize("dtype,kernel,opA,opB,m,n,k", NESTED_CASES)
def test_sb_gemm_nested_four_levels_in_one_launch(dtype, kernel, opA, opB, m, n, k):
    # section III-F with four batched modes and no loop on the host: levels whose strides do not nest in any
    # tensor (C's levels are laid out in another order than they are counted, A skips two of them, B one),
    # through every kernel family that decodes deep nests, against Listing 1 applied per outer index
    cnt = [3, 2, 4, 2]
    rng = np.random.default_rng(m + n + k)
    lda = (m if opA == "N" else k) + 1
    ldb = (k if opB == "N" else n) + 2
    ldc = m + 3
    sizeA, sizeB, sizeC = lda * (k if opA == "N" else m), ldb * (n if opB == "N" else k), ldc * n
    # C: level order 2, 0, 3, 1 from the inside out, with a little padding
    sC, step = [0] * 4, sizeC + 5
    for l in (2, 0, 3, 1):
        sC[l] = step
        step = step * cnt[l] + 7
    sA = [sizeA + 3, 0, (sizeA + 3) * cnt[0], 0]                     # A moves with levels 0 and 2 only
    sB = [0, sizeB, sizeB * cnt[1] + 11, (sizeB * cnt[1] + 11) * cnt[2]]     # B ignores level 0
    span = lambda s, size: size + sum(si * (c - 1) for si, c in zip(s, cnt)) + 3
    a = quantise(rng.uniform(-1, 1, span(sA, sizeA)), dtype)
    b = quantise(rng.uniform(-1, 1, span(sB, sizeB)), dtype)
    c0 = quantise(rng.uniform(-1, 1, span(sC, sizeC)), dtype)
    dA, dB, dC = to_dev(a, dtype), to_dev(b, dtype), to_dev(c0, dtype)
    alpha, beta = 0.75, -0.5
    sb.sb_force_kernel(KERNELS[kernel])
    sb.sb_gemm_nested(opA, opB, m, n, k, alpha, dA, lda, sA, dB, ldb, sB, beta, dC, ldc, sC, cnt, dt=dtype)
    sync()
    if kernel != "auto":
        assert sb.sb_last_kernel() == KERNELS[kernel]
    ref = c0.copy()
    inside = np.zeros(c0.size, dtype=bool)
    for p1, p2, p3 in itertools.product(range(cnt[1]), range(cnt[2]), range(cnt[3])):
        oa, ob, oc = (p1 * s[1] + p2 * s[2] + p3 * s[3] for s in (sA, sB, sC))
        part = oracle.sb_gemm(opA, opB, m, n, k, alpha, a[oa:], lda, sA[0], b[ob:], ldb, sB[0], beta, c0[oc:], ldc, sC[0], cnt[0],
                              wide=(dtype == "f64"))
        window = gemm_window_mask(c0.size - oc, m, n, ldc, sC[0], cnt[0])
        ref[oc:][window] = part[window]
        inside[oc:] |= window
    got = from_dev(dC)
    assert np.array_equal(got[~inside], c0[~inside]), "elements outside the m x n windows were written"
    assert_close(got[inside], ref[inside], dtype, k, 1.0, 1.0, alpha, beta, c0[inside], what=(dtype, kernel, opA, opB, m, n, k))


def test_extended_operations_directly():
    # section III-E: sb_gemm(OP_EX_N, OP_T, M, N, K, 1, B, ldb<1>, ldb<2>, A, lda<1>, 0, 0, C, ldc<1>, ldc<2>, P)
    M, N, P, K = 40, 30, 17, 23
    A = inputs.uniform_tensor(1, [N, K], np.float32)          # A_nk
    B = inputs.uniform_tensor(2, [P, M, K], np.float32)       # B_pmk  (case 3.6)
    tA, tB = to_dev(A, "f32"), to_dev(B, "f32")
    tC = to_dev(np.zeros(M * N * P), "f32")
    sb.sb_gemm("EX_N", "T", M, N, K, 1.0, tB, P, P * M, tA, N, 0, 0.0, tC, M, M * N, P, dt="f32")
    sync()
    ref = oracle.contract("nk", A, "pmk", B, "mnp", wide=False)
    assert_close(from_dev(tC, [M, N, P]), ref, "f32", K, 1.0, 1.0, what="case 3.6")
    # case 6.4: sb_gemm(OP_EX_T, OP_N, M, P, K, 1, B, ldb<1>, ldb<2>, A, lda<1>, 0, 0, C, ldc<2>, ldc<1>, N)
    A = inputs.uniform_tensor(3, [K, P], np.float32)          # A_kp
    B = inputs.uniform_tensor(4, [N, K, M], np.float32)       # B_nkm
    tA, tB = to_dev(A, "f32"), to_dev(B, "f32")
    tC = to_dev(np.zeros(M * N * P), "f32")
    sb.sb_gemm("EX_T", "N", M, P, K, 1.0, tB, N, N * K, tA, K, 0, 0.0, tC, M * N, M, N, dt="f32")
    sync()
    ref = oracle.contract("kp", A, "nkm", B, "mnp", wide=False)
    assert_close(from_dev(tC, [M, N, P]), ref, "f32", K, 1.0, 1.0, what="case 6.4")


EX_FORMS = [("EX_N", "N"), ("EX_N", "T"), ("EX_T", "N"), ("EX_T", "T"), ("N", "EX_N"), ("T", "EX_N"), ("N", "EX_T"), ("T", "EX_T")]


@pytest.mark.parametrize("dtype", ["f64", "f32", "bf16"])
@pytest.mark.parametrize("kernel", ["mfma", "generic", "auto"])
@pytest.mark.parametrize("opA,opB", EX_FORMS)
def test_extended_operation_on_either_operand(dtype, kernel, opA, opB):
    # section III-E on the first or on the second operand: the extended operand is a [P][rows][cols]
    # (or [P][cols][rows]) tensor with padded leading extent, batched in its unit-stride mode; the
    # other operand is a plain matrix shared by all batches; beta reads C; shapes span several bricks
    # (16 batches x 16 rows) with ragged tails.  The MFMA family must take every form itself.
    for (m, n, k, P, alpha, beta) in [(40, 30, 23, 17, 0.75, -0.5), (70, 130, 33, 37, 1.0, 0.0), (16, 16, 8, 8, -1.0, 1.0)]:
        rng = np.random.default_rng(m + n)

        def operand(op, rows, cols):             # op(X) is rows x cols; returns (ld, stride0, size)
            if op in ("N", "T"):
                r, c = (rows, cols) if op == "N" else (cols, rows)
                return r + 2, 0, (r + 2) * c + 3
            inner, outer = (rows, cols) if op == "EX_N" else (cols, rows)     # EX_N: rows next to the batch mode
            ld = P + 1
            return ld, ld * inner + 5, (ld * inner + 5) * outer + 3

        lda, sA, sizeA = operand(opA, m, k)
        ldb, sB, sizeB = operand(opB, k, n)
        ldc, sC = m + 3, (m + 3) * n + 1
        a = quantise(rng.uniform(-1, 1, sizeA), dtype)
        b = quantise(rng.uniform(-1, 1, sizeB), dtype)
        c0 = quantise(rng.uniform(-1, 1, sC * P + 2), dtype)
        dA, dB, dC = to_dev(a, dtype), to_dev(b, dtype), to_dev(c0, dtype)
        sb.sb_force_kernel(KERNELS[kernel])
        sb.sb_gemm(opA, opB, m, n, k, alpha, dA, lda, sA, dB, ldb, sB, beta, dC, ldc, sC, P, dt=dtype)
        sync()
        if kernel != "auto":
            assert sb.sb_last_kernel() == KERNELS[kernel], (kernel, sb.sb_last_kernel(), opA, opB, m, n, k, P)

        def packed(x, op, rows, cols, ld, s0):   # the P matrices op(X_b), gathered into packed column-major copies
            rs, cs, bs = {"N": (1, ld, s0), "T": (ld, 1, s0), "EX_N": (ld, s0, 1), "EX_T": (s0, ld, 1)}[op]
            bb, jj, ii = np.meshgrid(np.arange(P), np.arange(cols), np.arange(rows), indexing="ij")
            return x[bb * bs + ii * rs + jj * cs].ravel()

        ref = oracle.sb_gemm("N", "N", m, n, k, alpha, packed(a, opA, m, k, lda, sA), m, m * k,
                             packed(b, opB, k, n, ldb, sB), k, k * n, beta, c0, ldc, sC, P, wide=(dtype == "f64"))
        got = from_dev(dC)
        inside = gemm_window_mask(got.size, m, n, ldc, sC, P)
        assert np.array_equal(got[~inside], c0[~inside]), "elements outside the m x n windows were written"
        assert_close(got[inside], ref[inside], dtype, k, 1.0, 1.0, alpha, beta, c0[inside], what=(dtype, kernel, opA, opB, m, n, k, P))
    sb.sb_force_kernel(KERNELS["auto"])


@pytest.mark.parametrize("dtype", ["f32", "f64"])
@pytest.mark.parametrize("opA,opB", EX_FORMS)
def test_extended_operation_members(opA, opB, dtype):
    # the members of the extended-operation kernel on whole bricks (16 batches x 16 rows x 64 columns, 64 bytes of
    # k): in fp32 and fp64 the direct-to-LDS member when every load is 16-byte aligned (leading extent padded by 4), the
    # register-staged bricks otherwise (padded by 1); quarter-size tiles when the large ones are few; either
    # operand, both orientations of the plain one, alpha and beta
    ex_first = opA.startswith("EX")
    for (m, n, k, P, pad, alpha, beta, member) in [
            (128, 128, 32, 128, 4, 1.0, 0.0, sb.SB_MEMBER_MFMA_EX_DMA), (128, 128, 48, 128, 0, 0.75, -0.5, sb.SB_MEMBER_MFMA_EX_DMA),
            (64, 256, 16, 256, 4, -1.0, 0.0, sb.SB_MEMBER_MFMA_EX_DMA), (256, 64, 80, 256, 0, 1.0, 1.0, sb.SB_MEMBER_MFMA_EX_DMA),
            (512, 512, 32, 128, 4, 0.5, 0.25, sb.SB_MEMBER_MFMA_EX_DMA),          # enough tiles for the 128-column ones
            (128, 128, 32, 128, 1, 1.0, 0.0, sb.SB_MEMBER_MFMA_EX_BRICK), (64, 64, 32, 64, 0, 1.0, 0.0, sb.SB_MEMBER_MFMA_EX_SMALL)]:
        # (64, 256) / (256, 64): whole bricks for one operand position only (16 rows of the extended operand, 64 of the other)
        rows_ex, rows_other = (m, n) if ex_first else (n, m)
        if member == sb.SB_MEMBER_MFMA_EX_DMA and (rows_ex % 16 or rows_other % 64):
            continue
        rng = np.random.default_rng(m + n + k)

        def operand(op, rows, cols):             # op(X) is rows x cols; returns (ld, stride0, size)
            if op in ("N", "T"):
                r, c = (rows, cols) if op == "N" else (cols, rows)
                return r + pad, 0, (r + pad) * c
            inner, outer = (rows, cols) if op == "EX_N" else (cols, rows)     # EX_N: rows next to the batch mode
            ld = P + pad
            return ld, ld * inner + 4 * pad, (ld * inner + 4 * pad) * outer

        lda, sA, sizeA = operand(opA, m, k)
        ldb, sB, sizeB = operand(opB, k, n)
        ldc, sC = m + pad, (m + pad) * n + pad
        a = quantise(rng.uniform(-1, 1, sizeA), dtype)
        b = quantise(rng.uniform(-1, 1, sizeB), dtype)
        c0 = quantise(rng.uniform(-1, 1, sC * P), dtype)
        dA, dB, dC = to_dev(a, dtype), to_dev(b, dtype), to_dev(c0, dtype)
        sb.sb_gemm(opA, opB, m, n, k, alpha, dA, lda, sA, dB, ldb, sB, beta, dC, ldc, sC, P, dt=dtype)
        sync()
        assert sb.sb_last_kernel() == sb.SB_KERNEL_MFMA and sb.sb_last_kernel_member() == member, \
            (opA, opB, m, n, k, P, pad, sb.sb_last_kernel(), sb.sb_last_kernel_member(), member)

        def packed(x, op, rows, cols, ld, s0):   # the P matrices op(X_b), gathered into packed column-major copies
            rs, cs, bs = {"N": (1, ld, s0), "T": (ld, 1, s0), "EX_N": (ld, s0, 1), "EX_T": (s0, ld, 1)}[op]
            bb, jj, ii = np.meshgrid(np.arange(P), np.arange(cols), np.arange(rows), indexing="ij")
            return x[bb * bs + ii * rs + jj * cs].ravel()

        ref = oracle.sb_gemm("N", "N", m, n, k, alpha, packed(a, opA, m, k, lda, sA), m, m * k,
                             packed(b, opB, k, n, ldb, sB), k, k * n, beta, c0, ldc, sC, P, wide=(dtype == "f64"))
        got = from_dev(dC)
        inside = gemm_window_mask(got.size, m, n, ldc, sC, P)
        assert np.array_equal(got[~inside], c0[~inside]), "elements outside the m x n windows were written"
        assert_close(got[inside], ref[inside], dtype, k, 1.0, 1.0, alpha, beta, c0[inside], what=(dtype, opA, opB, m, n, k, P, pad))


def test_runs_on_a_side_stream():
    import torch
    s = torch.cuda.Stream()
    A = inputs.uniform_tensor(1, [48, 40], np.float32)
    B = inputs.uniform_tensor(2, [40, 24, 9], np.float32)
    tA, tB = to_dev(A, "f32"), to_dev(B, "f32")
    tC = to_dev(np.zeros(48 * 24 * 9), "f32")
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        sb.sb_contract("mk", "knp", "mnp", 1.0, tA, [48, 40], tB, [40, 24, 9], 0.0, tC)
    s.synchronize()
    ref = oracle.contract("mk", A, "knp", B, "mnp", wide=False)
    assert_close(from_dev(tC, [48, 24, 9]), ref, "f32", 40, 1.0, 1.0)


@pytest.mark.parametrize("dtype", ["f64", "f32", "bf16"])
def test_mode_permutation_is_exact(dtype):
    # sb_permute (the copy step of the conventional evaluation, used by the benchmark's baseline) moves
    # bits: every permutation of an order-3 tensor with ragged extents, some of order 2 and 4
    import torch
    cases = [((70, 33, 129), p) for p in itertools.permutations(range(3))]
    cases += [((300, 77), (1, 0)), ((5, 1, 66, 9), (2, 0, 3, 1)), ((64, 64, 64), (1, 0, 2)), ((4100,), (0,)), ((3, 4, 5, 6), (3, 2, 1, 0))]
    for dims, perm in cases:
        X = inputs.make_tensor(77, list(dims), dtype)
        tX = to_dev(X, dtype)
        tY = torch.zeros_like(tX)
        sb.sb_permute(dims, perm, tX, tY, dt=dtype)
        sync()
        want = np.transpose(quantise(X, dtype), perm)
        got = from_dev(tY, want.shape)
        assert np.array_equal(got, want), (dims, perm)


def test_plan_cache_alternating_contractions():
    # sb_contract keeps the plans of the last eight distinct contractions per thread: ten different
    # ones in rotation (more than the cache holds, so entries are evicted and re-planned), same
    # results with the cache switched off, and a changed extent under the same mode strings must not
    # find the old plan
    cases = cases_2x3()[::4][:9] + [("mk", "knp")]
    try:
        for enabled in (True, False, True):
            sb.sb_plan_cache_enable(enabled)
            for rnd in range(3):
                for i, (ma, mb) in enumerate(cases):
                    ext = dict(m=24 + i, n=9, p=5, k=7 + rnd)        # k changes from round to round
                    contract_case("f32", ma, mb, "mnp", ext, alpha=1.5, beta=0.5, seed=600 + i)
    finally:
        sb.sb_plan_cache_enable(True)


def test_general_orders_sampled():
    # the planner's procedure is the same for any order (Algorithm 2): a sample of the 216 order-3 x
    # order-3 cases, and order 4 x 2 / 2 x 4 / 4 x 3 contractions with C in scrambled mode order
    from helpers import cases_general
    ext = dict(m=20, n=9, p=12, q=7, r=5, k=17)
    cases = cases_general(3, 3)[::9]
    cases += [("mkpq", "nk", "qnmp"), ("km", "qknp", "npmq"), ("pmkq", "rkn", "mqrnp"), ("qpkm", "nrk", "pmnqr")]
    for i, (ma, mb, mc) in enumerate(cases):
        for strat in ("auto", "nested"):
            err, text = contract_case("f32", ma, mb, mc, ext, strat=strat, alpha=1.25, beta=0.5, seed=300 + i)
            assert err <= TOL["f32"], (ma, mb, mc, strat, text, err)


@pytest.mark.parametrize("dtype", ["f64", "f32", "bf16"])
def test_vector_operands(dtype):
    # the level-2 and level-1 rows of Table I through sb_contract: matrix-vector products in both
    # storage orders, tensor-vector products batched over the last mode, flattened, and with the
    # extended operation (batch over the first mode);
    # large enough for several workgroups of the thin kernels, with ragged extents
    ext = dict(m=1030, n=6, p=37, k=531)
    for i, (ma, mb, mc) in enumerate([("mk", "k", "m"), ("km", "k", "m"), ("mkp", "k", "mp"), ("kmp", "k", "mp"),
                                      ("pkm", "k", "mp"), ("k", "km", "m")]):
        err, text = contract_case(dtype, ma, mb, mc, ext, alpha=1.5, beta=-0.25, seed=500 + i)
        assert err <= TOL[dtype], (ma, mb, mc, text, err)
        assert sb.sb_last_kernel() == sb.SB_KERNEL_THIN, (ma, mb, mc, text)


def test_replays_inside_a_hip_graph():
    # the library allocates nothing and never synchronises, so a sequence of contractions can be
    # captured once and replayed; every replay is checked, with eager work between the replays
    import torch
    ext = dict(m=48, n=40, p=9, k=24)
    A = inputs.uniform_tensor(1, [ext["k"], ext["m"]], np.float32)
    B = inputs.uniform_tensor(2, [ext["k"], ext["n"], ext["p"]], np.float32)
    tA, tB = to_dev(A, "f32"), to_dev(B, "f32")
    tC = to_dev(np.zeros(ext["m"] * ext["n"] * ext["p"]), "f32")
    tD = to_dev(np.zeros(ext["k"] * ext["n"] * ext["p"]), "f32")
    dA, dB = [ext["k"], ext["m"]], [ext["k"], ext["n"], ext["p"]]

    def work():
        sb.sb_contract("km", "knp", "mnp", 1.0, tA, dA, tB, dB, 0.0, tC)                                   # C_mnp
        sb.sb_contract("ms", "mnp", "snp", 2.0, tA, [ext["m"], ext["k"]], tC, [ext["m"], ext["n"], ext["p"]], 0.0, tD)

    A2 = A.reshape(-1, order="F")[: ext["m"] * ext["k"]].reshape([ext["m"], ext["k"]], order="F")
    ref_c = oracle.contract("km", A, "knp", B, "mnp", wide=False)
    ref_d = oracle.contract("ms", A2, "mnp", ref_c, "snp", alpha=2.0, wide=False)
    work()                                   # warm-up outside the capture (first-use set-up of the kernels)
    sync()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            work()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(4):
        tC.fill_(float("nan"))
        tD.fill_(float("nan"))
        sync()
        graph.replay()
        sync()
        assert_close(from_dev(tC, ref_c.shape), ref_c, "f32", ext["k"], 1.0, 1.0, what=rep)
        # the second contraction consumes the device's own (rounded) C: bound its inputs' error too
        assert_close(from_dev(tD, [ext["k"], ext["n"], ext["p"]]), ref_d, "f32", 2 * ext["m"], 1.0, np.abs(ref_c).max(), 2.0,
                     what=rep)
        tB.mul_(1.0)                         # eager work between replays


def test_replays_of_the_wide_block_and_block_split_members_inside_a_hip_graph():
    # the same for the members that count their own outstanding loads and stores (wide-block panel kernel)
    # or re-describe the batch (tiny kernel's 16 x 16 blocks): a nested bf16 product and a short fp64 batch
    import torch
    e5 = dict(m=64, n=64, p=4, q=8, k=128)
    A5 = inputs.make_tensor(21, [e5["m"], e5["p"], e5["k"]], "bf16")
    B5 = inputs.make_tensor(22, [e5["k"], e5["n"], e5["q"]], "bf16")
    e1 = dict(m=32, n=32, p=8, k=32)
    A1 = inputs.uniform_tensor(23, [e1["m"], e1["k"]])
    B1 = inputs.uniform_tensor(24, [e1["k"], e1["n"], e1["p"]])
    tA5, tB5, tA1, tB1 = to_dev(A5, "bf16"), to_dev(B5, "bf16"), to_dev(A1, "f64"), to_dev(B1, "f64")
    d5, d1 = [e5[c] for c in "mpnq"], [e1[c] for c in "mnp"]
    tC5 = to_dev(np.zeros(int(np.prod(d5))), "bf16")
    tC1 = to_dev(np.zeros(int(np.prod(d1))), "f64")

    def work():
        sb.sb_force_kernel(sb.SB_KERNEL_PANEL)       # two blocks only: the selector would take 64 x 64 tiles
        sb.sb_contract("m[p]k", "kn[q]", "m[p]n[q]", 1.0, tA5, list(A5.shape), tB5, list(B5.shape), 0.0, tC5, d5, dt="bf16")
        sb.sb_force_kernel(sb.SB_KERNEL_AUTO)
        sb.sb_contract("mk", "kn[p]", "mn[p]", 1.0, tA1, list(A1.shape), tB1, list(B1.shape), 0.0, tC1, d1, dt="f64")

    ref5 = oracle.contract("mpk", A5, "knq", B5, "mpnq", wide=False)
    ref1 = oracle.contract("mk", A1, "knp", B1, "mnp", wide=True)
    work()                                   # warm-up outside the capture; and the members are the intended ones
    sync()
    assert sb.sb_last_kernel() == sb.SB_KERNEL_TINY and sb.sb_last_kernel_member() == sb.SB_MEMBER_TINY_BLOCKS
    sb.sb_force_kernel(sb.SB_KERNEL_PANEL)
    sb.sb_contract("m[p]k", "kn[q]", "m[p]n[q]", 1.0, tA5, list(A5.shape), tB5, list(B5.shape), 0.0, tC5, d5, dt="bf16")
    sync()
    assert sb.sb_last_kernel() == sb.SB_KERNEL_PANEL and sb.sb_last_kernel_member() == sb.SB_MEMBER_PANEL_WIDE
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            work()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(4):
        tC5.fill_(float("nan"))
        tC1.fill_(float("nan"))
        sync()
        graph.replay()
        sync()
        assert_close(from_dev(tC5, d5), ref5, "bf16", e5["k"], np.abs(A5).max(), np.abs(B5).max(), what=rep)
        assert_close(from_dev(tC1, d1), ref1, "f64", e1["k"], 1.0, 1.0, what=rep)
        tB1.mul_(1.0)                        # eager work between replays


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("opA,opB", [("N", "N"), ("T", "N"), ("N", "T"), ("T", "T")])
def test_sb_gemm_whole_tile_shapes(dtype, opA, opB):
    # whole 128 x 128 (or 64 x 64) tiles with k a multiple of 32: the streaming member of the MFMA
    # family, whose panel stream runs across tile boundaries; shortest legal k, odd tile counts,
    # more and fewer tiles than resident workgroups, beta = 0 and beta != 0 (separate kernels)
    # of the last five, two fill the chip with 128 x 256 tiles and two with 256 x 256 tiles (the eight-wave fp32
    # configurations); the one between them would leave a round mostly empty with either and stays on 128 x 128
    for m, n, k, batch in ((256, 384, 64, 5), (256, 384, 64, 30), (128, 128, 96, 3), (64, 192, 160, 7), (512, 256, 64, 37), (128, 256, 512, 1),
                           (384, 512, 96, 128), (128, 256, 160, 512), (384, 256, 64, 260), (256, 256, 64, 256), (512, 256, 96, 128),
                           # whole tiles with k a multiple of 64: the members that load straight into LDS, in fp32 on 128 x 256
                           # tiles (6 and 4 panels of 32) and, with k >= 256 and two rounds of tiles, on 256 x 256 tiles
                           (256, 256, 192, 256), (512, 512, 128, 128), (256, 256, 256, 512),
                           # the same member on 128 x 128 tiles (8 panels) and, in fp32, on 128 x 256 tiles (4 panels)
                           (128, 384, 256, 60), (128, 512, 128, 200)):
        lda = (m if opA == "N" else k) + 4
        ldb = (k if opB == "N" else n) + 8
        ldc = m + 12
        loa = lda * (k if opA == "N" else m) + 16
        lob = ldb * (n if opB == "N" else k)
        loc = ldc * n + 4
        for alpha, beta in ((1.0, 0.0), (-0.5, 1.5)):
            err, got, ref = run_sb_gemm(dtype, opA, opB, m, n, k, batch, lda, ldb, ldc, loa, lob, loc, alpha, beta,
                                        seed=m + n + k, kernel="mfma")
            assert err <= TOL[dtype], (m, n, k, batch, alpha, beta, err)


def test_sb_gemm_whole_tile_shapes_bf16():
    # bf16 with both operands k-contiguous, whole 128 x 128 tiles, k a multiple of 128 (at least 256):
    # the streaming bf16 kernel; shortest legal k, odd tile counts, more and fewer tiles than resident
    # workgroups, beta = 0 and beta != 0 (separate kernels).  The neighbouring shapes (k = 320, an
    # operand not k-contiguous) take the plain bf16 kernel and are checked the same way.  The last
    # three fill the chip with 256 x 256 tiles: the eight-wave variant (k a multiple of 64).
    for opA, opB, m, n, k, batch in (("T", "N", 256, 384, 256, 5), ("T", "N", 128, 128, 384, 3), ("T", "N", 128, 256, 1024, 1),
                                     ("T", "N", 512, 256, 256, 131), ("T", "N", 128, 128, 320, 3), ("N", "N", 256, 128, 256, 2),
                                     ("T", "N", 512, 768, 128, 128), ("T", "N", 1024, 512, 1088, 32), ("T", "N", 256, 256, 192, 256),
                                     # k a multiple of 128: the 256 x 256 member that loads straight into LDS (2, 6 and 10 panels of 64;
                                     # more tiles than workgroups, so the panel stream crosses tile boundaries)
                                     ("T", "N", 512, 512, 384, 128), ("T", "N", 256, 768, 640, 170),
                                     # the same member with row-contiguous operands (kept [k][row] in LDS, transposed by the fragment reads)
                                     ("N", "T", 512, 512, 384, 128), ("T", "T", 256, 768, 256, 170), ("N", "N", 768, 256, 128, 171),
                                     # operands with m or n contiguous are transposed on their way into LDS: the same
                                     # streaming kernels in the other three layouts, 128 x 128 and 256 x 256 tiles
                                     ("N", "N", 256, 384, 256, 5), ("N", "T", 128, 256, 384, 3), ("T", "T", 384, 128, 512, 2),
                                     ("N", "N", 512, 768, 128, 128), ("N", "T", 256, 256, 192, 256), ("T", "T", 512, 512, 256, 70)):
        lda = (m if opA == "N" else k) + 8
        ldb = (k if opB == "N" else n) + 16
        ldc = m + 12
        loa = lda * (k if opA == "N" else m) + 16
        lob = ldb * (n if opB == "N" else k)
        loc = ldc * n + 4
        for alpha, beta in ((1.0, 0.0), (-0.5, 1.5)):
            err, got, ref = run_sb_gemm("bf16", opA, opB, m, n, k, batch, lda, ldb, ldc, loa, lob, loc, alpha, beta,
                                        seed=m + n + k, kernel="mfma")
            assert err <= TOL["bf16"], (opA, opB, m, n, k, batch, alpha, beta, err)


def test_offsets_beyond_2_31_elements():
    # tensors with more than 2^31 elements (8.7 GB each in fp32): 64-bit offsets in the tiny-matrix and
    # the MFMA kernels, millions of batches.  B is a seeded vector of prime length repeated along memory,
    # so the host can rebuild any column; sampled columns of C (the last ones, the ones around element
    # 2^31, random ones) are compared with the oracle, and no element of C may be left unwritten.
    import torch
    L = 1000003
    base = inputs.uniform_tensor(123, [L], np.float32)
    base_dev = to_dev(base, "f32")
    rng = np.random.default_rng(7)
    for m, n, k, p in ((16, 16, 16, 8_500_000), (64, 64, 64, 530_000)):
        total = k * n * p
        assert total > 2 ** 31
        tB = torch.empty(total, dtype=torch.float32, device="cuda")
        chunk = 1 << 27
        for s0 in range(0, total, chunk):
            idx = torch.arange(s0, min(s0 + chunk, total), device="cuda") % L
            tB[s0:s0 + idx.numel()] = base_dev[idx]
        del idx
        A = inputs.uniform_tensor(124, [m, k], np.float32)
        tA = to_dev(A, "f32")
        tC = torch.full((m * n * p,), float("nan"), dtype=torch.float32, device="cuda")
        sb.sb_contract("mk", "knp", "mnp", 1.0, tA, [m, k], tB, [k, n, p], 0.0, tC, [m, n, p])
        sync()
        assert not bool(torch.isnan(tC).any())
        edge = 2 ** 31 // (k * n)
        for pp in [int(x) for x in rng.integers(0, p, 12)] + [p - 1, p - 2, edge - 1, edge, edge + 1, 0]:
            for nn in (0, n - 1, int(rng.integers(0, n))):
                off = k * nn + k * n * pp
                col = base[(off + np.arange(k)) % L]
                ref = oracle.contract("mk", A, "k", col, "m", wide=False)
                got = tC[m * nn + m * n * pp: m * nn + m * n * pp + m].cpu().numpy().astype(np.float64)
                assert_close(got, ref, "f32", k, 1.0, 1.0, what=(m, pp, nn))
        del tB, tC
        torch.cuda.empty_cache()


def test_thin_kernels_beyond_2_31_elements():
    # one matrix of more than 2^31 elements (8.7 GB in fp32) times a vector, in both layouts: 64-bit
    # offsets in the rows and the dots kernel.  The matrix is a seeded vector of prime length repeated
    # along memory, so the host can rebuild any row; sampled entries of y (first, last, the ones whose
    # row crosses element 2^31, random ones) are compared with the oracle, none may be left unwritten.
    import torch
    L = 1000003
    base = inputs.uniform_tensor(125, [L], np.float32)
    base_dev = to_dev(base, "f32")
    rng = np.random.default_rng(8)
    rows, k = 1 << 22, 520
    total = rows * k
    assert total > 2 ** 31
    tA = torch.empty(total, dtype=torch.float32, device="cuda")
    chunk = 1 << 27
    for s0 in range(0, total, chunk):
        idx = torch.arange(s0, min(s0 + chunk, total), device="cuda") % L
        tA[s0:s0 + idx.numel()] = base_dev[idx]
    del idx
    x = inputs.uniform_tensor(126, [k], np.float32)
    tx = to_dev(x, "f32")
    for op in ("N", "T"):
        ty = torch.full((rows,), float("nan"), dtype=torch.float32, device="cuda")
        lda = rows if op == "N" else k
        sb.sb_gemm(op, "N", rows, 1, k, 1.0, tA, lda, 0, tx, k, 0, 0.0, ty, rows, 0, 1, dt="f32")
        sync()
        assert sb.sb_last_kernel() == sb.SB_KERNEL_THIN
        assert not bool(torch.isnan(ty).any())
        edge = 2 ** 31 // k if op == "T" else 2 ** 31 % rows
        sample = [int(v) for v in rng.integers(0, rows, 24)] + [0, 1, rows - 1, rows - 2] + \
                 [e for e in (edge - 1, edge, edge + 1) if 0 <= e < rows]
        l = np.arange(k)
        M = np.stack([base[((i + l * rows) if op == "N" else (l + i * k)) % L] for i in sample])
        ref = oracle.contract("mk", M, "k", x, "m", wide=False)
        got = ty[torch.tensor(sample, device="cuda")].cpu().numpy().astype(np.float64)
        assert_close(got, ref, "f32", k, 1.0, 1.0, what=op)
        del ty
    del tA
    torch.cuda.empty_cache()
