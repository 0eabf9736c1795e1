"""The C-ABI library loads, exports every declared symbol, and validates arguments on the host
(no test here launches a kernel, so this module runs without a GPU)."""
import os
import re

import paper_1606_05696_amd as sb
from paper_1606_05696_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000      # never dereferenced: validation fails (or the problem is empty) before any launch


def declared_functions():
    names = []
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"^(?:int|int64_t|const char \*)\s*(sb_\w+)\s*\(", text, flags=re.M)
    return names


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert set(names) >= {"sb_gemm", "sb_gemm2", "sb_contract", "sb_contract_plan", "sb_plan_launch", "sb_plan_launches",
                          "sb_status_string", "sb_force_kernel", "sb_last_kernel", "sb_select_kernel", "sb_tucker_workspace",
                          "sb_tucker_hooi", "sb_sym_eig_workspace", "sb_sym_eig", "sb_probe_mfma"}
    lib = binding.load()
    for n in names:
        assert getattr(lib, n) is not None
        assert hasattr(binding, n), "the Python binding must expose %s under the same name" % n


def gemm(**over):
    a = dict(dt=sb.SB_F32, transA="N", transB="N", m=4, n=5, k=6, alpha=1.0, A=FAKE, lda=4, strideA=0,
             B=FAKE, ldb=6, strideB=30, beta=0.0, C=FAKE, ldc=4, strideC=20, batch=3)
    a.update(over)
    return sb.sb_gemm(a["transA"], a["transB"], a["m"], a["n"], a["k"], a["alpha"], a["A"], a["lda"], a["strideA"],
                      a["B"], a["ldb"], a["strideB"], a["beta"], a["C"], a["ldc"], a["strideC"], a["batch"],
                      dt=a["dt"], stream=0, check=False)


def test_sb_gemm_argument_validation():
    assert gemm(dt=7) == -1
    assert gemm(transA=9) == -2
    assert gemm(transB=-1) == -3
    assert gemm(m=-1) == -4
    assert gemm(n=-1) == -5
    assert gemm(k=-1) == -6
    assert gemm(A=None) == -8
    assert gemm(lda=3) == -9                      # N: lda >= m
    assert gemm(transA="T", lda=5) == -9          # T: lda >= k
    assert gemm(strideA=-1) == -10
    assert gemm(B=None) == -11
    assert gemm(ldb=5) == -12                     # N: ldb >= k
    assert gemm(transB="T", ldb=4) == -12         # T: ldb >= n
    assert gemm(strideB=-2) == -13
    assert gemm(C=None) == -15
    assert gemm(ldc=3) == -16
    assert gemm(strideC=0) == -17                 # batches of C would coincide
    assert gemm(strideC=-4) == -17
    assert gemm(batch=-1) == -18
    # batches of C that overlap without coinciding: 4 x 5 windows (20 elements) only 19 or 7 apart
    assert gemm(strideC=19) == -17
    assert gemm(strideC=7) == -17
    assert gemm(ldc=6, strideC=25) == -17          # columns 6 apart: a batch spans 28 elements
    assert gemm(m=1, n=5, ldc=3, strideC=2, batch=3) == -16      # sorted by stride, ldc is the one that is too small
    assert gemm(transA="EX_N", strideA=0) == -10  # extended op: the stride argument is a column stride
    # quick returns: nothing to do, nothing launched
    assert gemm(m=0) == sb.SB_OK
    assert gemm(n=0) == sb.SB_OK
    assert gemm(batch=0) == sb.SB_OK
    assert gemm(batch=0, C=None) == sb.SB_OK


def test_sb_gemm2_argument_validation():
    def g2(**over):
        a = dict(sA0=0, sA1=0, sB0=30, sB1=90, sC0=20, sC1=60, b0=3, b1=2, lda=4, ldb=6, ldc=4)
        a.update(over)
        return sb.sb_gemm2("N", "N", 4, 5, 6, 1.0, FAKE, a["lda"], a["sA0"], a["sA1"], FAKE, a["ldb"], a["sB0"], a["sB1"],
                           0.0, FAKE, a["ldc"], a["sC0"], a["sC1"], a["b0"], a["b1"], dt=sb.SB_F64, stream=0, check=False)
    assert g2(sA1=-1) == -11
    assert g2(sB1=-1) == -15
    assert g2(sC0=0) == -19
    assert g2(sC1=0) == -20
    assert g2(b0=-1) == -21
    assert g2(b1=-1) == -22
    assert g2(ldc=2) == -18
    assert g2(sC0=19) == -19                       # level-0 batches overlap
    assert g2(sC1=59) == -20                       # level-1 batches overlap (three level-0 batches span 60)
    assert g2(b1=0) == sb.SB_OK


def test_sb_gemm_nested_argument_validation():
    def gn(**over):
        a = dict(sA=[0, 0, 0], sB=[30, 90, 180], sC=[20, 60, 120], cnt=[3, 2, 2], lda=4, ldb=6, ldc=4, A=FAKE, B=FAKE, C=FAKE)
        a.update(over)
        return sb.sb_gemm_nested("N", "N", 4, 5, 6, 1.0, a["A"], a["lda"], a["sA"], a["B"], a["ldb"], a["sB"], 0.0, a["C"], a["ldc"],
                                 a["sC"], a["cnt"], dt=sb.SB_F32, stream=0, check=False)
    assert gn(sA=[0, -1, 0]) == -10
    assert gn(sB=[30, 90, -5]) == -13
    assert gn(sC=[20, 60, 0]) == -17                # two batches of level 2 coincide
    assert gn(sC=[20, 60, 119]) == -17              # ... or overlap
    assert gn(sC=[20, 59, 120]) == -17
    assert gn(cnt=[3, -2, 2]) == -19
    assert gn(ldc=3) == -16
    assert gn(C=None) == -15
    assert gn(cnt=[3, 0, 2]) == sb.SB_OK            # an empty level: nothing to do
    assert gn(cnt=[3, 2, 2, 1, 1, 1, 1, 1, 1], sA=[0] * 9, sB=[0] * 9, sC=[1] * 9) == -18     # more than SB_MAX_BATCH_LEVELS


def test_sb_contract_argument_validation():
    def c(**over):
        a = dict(dt=sb.SB_F32, A="mk", B="knp", C="mnp", dA=[4, 6], dB=[6, 5, 3], pa=FAKE, pb=FAKE, pc=FAKE, strat=0)
        a.update(over)
        return sb.sb_contract(a["A"], a["B"], a["C"], 1.0, a["pa"], a["dA"], a["pb"], a["dB"], 0.0, a["pc"],
                              strat=a["strat"], dt=a["dt"], stream=0, check=False)
    assert c(dt=5) == -1
    assert c(dA=None) == -7
    assert c(dB=None) == -10
    assert c(strat=17) == -16
    assert c(C="mn") == sb.SB_ERR_CONTRACTION
    assert c(A="m(k") == sb.SB_ERR_MODES
    assert c(pa=None) == -6
    assert c(pb=None) == -9
    assert c(pc=None) == -13
    assert c(A="nk", B="pkm", dA=[5, 6], dB=[3, 6, 4], strat=sb.SB_FLATTEN) == sb.SB_ERR_ILLEGAL_EVAL
    # an empty contraction needs no launch
    assert c(dA=[0, 6], dB=[6, 5, 3]) == sb.SB_OK


def test_sb_permute_argument_validation():
    perm = lambda dims=(4, 5, 6), p=(2, 0, 1), src=FAKE, dst=FAKE + 4096, dt="f32": \
        sb.sb_permute(list(dims), list(p), src, dst, dt=dt, stream=0, check=False)
    assert perm(dt=9) == -1
    assert perm(dims=(), p=()) == -2
    assert perm(dims=(4, -1, 6)) == -3
    assert perm(p=(0, 0, 1)) == -4 and perm(p=(0, 1, 3)) == -4
    assert perm(src=None) == -5
    assert perm(dst=None) == -6 and perm(dst=FAKE) == -6
    assert perm(dims=(4, 0, 6)) == sb.SB_OK            # empty tensor: nothing to do


def test_status_strings():
    assert sb.sb_status_string(0) == "success"
    for code in (-3, 1, 2, 3, 4, 5, 6, 1000 + 98):
        assert len(sb.sb_status_string(code)) > 5
    assert "launch" in sb.sb_status_string(1098)


def test_force_kernel_rejects_unknown_ids():
    assert sb.sb_force_kernel(12) == -1
    assert sb.sb_force_kernel(sb.SB_KERNEL_AUTO) == sb.SB_OK


def test_tucker_argument_validation_on_the_host():
    hooi = lambda dt="f32", dims=(4, 4, 4), core=(2, 2, 2), its=1, T=FAKE, ws=FAKE - FAKE % 256, nbytes=1 << 30: \
        binding.load().sb_tucker_hooi(binding.DTYPES[dt], T, *dims, *core, its, 1, FAKE, FAKE, FAKE, FAKE, ws, nbytes, None)
    assert hooi(dt="bf16") == -1
    assert hooi(T=None) == -2
    assert hooi(dims=(0, 4, 4)) == -3 and hooi(dims=(4, 0, 4)) == -4 and hooi(dims=(4, 4, 0)) == -5
    assert hooi(core=(5, 2, 2)) == -6 and hooi(core=(2, 5, 2)) == -7 and hooi(core=(2, 2, 5)) == -8
    assert hooi(core=(1, 1, 2)) == -8                    # k may not exceed i*j
    assert hooi(its=-1) == -9
    assert hooi(ws=None) == -15 and hooi(ws=FAKE + 8) == -15 and hooi(nbytes=64) == -16
    rc, need = sb.sb_tucker_workspace("f32", 256, 256, 256, 10, 10, 10, with_init=False)
    assert rc == 0 and need % 256 == 0
    # W1 (m n k), Z (i n p), Y, the selected eigenvectors, four 100 x 100 matrices, lambda, selection
    assert need >= 4 * (256 * 256 * 10 + 10 * 256 * 256 + 256 * 100 + 100 * 10 + 4 * 100 * 100 + 100) + 4 * 100
    assert sb.sb_tucker_workspace("f32", 256, 256, 256, 10, 10, 10, with_init=True)[1] >= need + 4 * 4 * (256 * 256 - 100 * 100)
    assert sb.sb_sym_eig_workspace("f64", 100)[1] >= 4 * 8 * 100 * 100
    assert sb.sb_sym_eig_workspace("f32", 5000, check=False)[0] == -2


def test_kernel_selector():
    """The selector is host arithmetic on shapes: each family gets the shapes it was built for."""
    def fam(dt, opA, opB, m, n, k, batch=8):
        lda = m if opA == "N" else k
        ldb = k if opB == "N" else n
        return sb.sb_select_kernel(dt, opA, opB, m, n, k, lda, m * k, ldb, k * n, m, m * n, batch)
    G, TINY, MFMA, THIN = sb.SB_KERNEL_GENERIC, sb.SB_KERNEL_TINY, sb.SB_KERNEL_MFMA, sb.SB_KERNEL_THIN
    for dt in ("f32", "f64"):
        assert fam(dt, "T", "N", 512, 512, 512) == MFMA            # the large cube
        assert fam(dt, "N", "N", 64, 64, 64) == MFMA               # the 36 cases at 64
        assert fam(dt, "N", "N", 16, 16, 16, 65536) == TINY        # the tiny-batch regime
        assert fam(dt, "N", "N", 32, 32, 32) == TINY
        assert fam(dt, "N", "N", 10, 10, 512, 512) == MFMA         # few small problems with a long k: the tiled kernels prefetch
        assert fam(dt, "N", "N", 10, 10, 512, 4096) == TINY        # many of them: one wavefront each
        assert fam(dt, "N", "N", 4096, 1, 4096) == THIN            # matrix-vector
        assert fam(dt, "N", "N", 1, 4096, 4096) == THIN            # vector-matrix
        assert fam(dt, "T", "N", 2048, 4, 100) == THIN
        assert fam(dt, "N", "N", 1, 1, 5) == TINY                  # short dot products stay with the small-matrix kernels
        assert fam(dt, "N", "N", 32, 1, 4096) == THIN              # long ones do not
        assert fam(dt, "T", "N", 16, 2, 512) == THIN               # rows contiguous along k
        assert fam(dt, "N", "N", 262144, 10, 512, 1) == MFMA       # factor matrix against an unfolding
        assert fam(dt, "N", "N", 100, 10, 100) == MFMA
        assert fam(dt, "N", "N", 100, 10, 16) == G                 # short k, mostly padding: vector-ALU kernel
        assert fam(dt, "N", "N", 33, 200, 1) == MFMA               # rank-1 updates: bound by writing C
    assert fam("bf16", "N", "N", 16, 16, 16) == MFMA
    assert fam("bf16", "N", "N", 100, 10, 16) == MFMA
    assert fam("bf16", "N", "N", 4096, 3, 64) == THIN
    # bf16 with k <= 128 and a large C: whole-k panels, blocks of 4 x 4 panels (the flattened form of the
    # order-3 x order-3 benchmark contraction, and its form batched over q with A shared)
    PANEL = sb.SB_KERNEL_PANEL
    assert fam("bf16", "N", "N", 4096, 4096, 128, 1) == PANEL
    assert sb.sb_select_kernel("bf16", "N", "N", 4096, 64, 128, 4096, 0, 128, 128 * 64, 4096, 4096 * 64, 64) == PANEL
    assert fam("bf16", "T", "T", 2048, 4096, 40, 1) == PANEL
    assert fam("bf16", "N", "N", 4096, 4096, 136, 1) == MFMA      # k too long for whole-k panels
    assert fam("bf16", "N", "N", 512, 512, 128, 1) == MFMA        # four blocks would use four compute units
    assert fam("bf16", "N", "N", 64, 64, 128, 4096) == MFMA       # every batch moves both operands: nothing to share
    assert fam("f32", "N", "N", 4096, 4096, 128, 1) == MFMA
    # extended operations (section III-E): on the first operand the MFMA family, on the second the general kernel
    # (with the second operand shared by the batches, as in the exceptional cases of Table II)
    assert sb.sb_select_kernel("f32", sb.SB_OP_EX_N, "N", 64, 64, 64, 64, 4096, 64, 0, 64, 4096, 8) == MFMA
    assert sb.sb_select_kernel("f32", "N", sb.SB_OP_EX_N, 64, 64, 64, 64, 4096, 64, 4096, 64, 4096, 8) == G
    assert sb.sb_select_kernel("f32", sb.SB_OP_EX_T, "N", 64, 1, 64, 64, 4096, 64, 4096, 64, 4096, 8) == THIN
    # argument checks
    assert sb.sb_select_kernel(7, "N", "N", 4, 4, 4, 4, 16, 4, 16, 4, 16, 1) == -1
    assert sb.sb_select_kernel("f32", "N", "N", 0, 4, 4, 4, 16, 4, 16, 4, 16, 1) == -4
    assert sb.sb_select_kernel("f32", "N", "N", 4, 4, 4, 4, 16, 4, 16, 3, 16, 1) == -11


def test_interleaved_batches_of_c_are_accepted_and_overlapping_ones_rejected():
    # sb_select_kernel validates C exactly as sb_gemm does and launches nothing.
    # C_m[n]p (Table II): m x p matrices with ldc = m*n, one per n, m apart -- legal although the
    # batch stride is far below ldc * columns
    m, n, p = 64, 48, 40
    sel = lambda ldc, sc, batch, rows=m, cols=p: sb.sb_select_kernel("f32", "N", "N", rows, cols, 16, rows, 0, 16, 16 * cols,
                                                                      ldc, sc, batch)
    assert sel(m * n, m, n) >= 0
    assert sel((m + 1) * n + 5, m + 1, n) >= 0         # padded: still disjoint
    assert sel(m * n, m - 1, n) == -12                 # neighbouring batches share a row
    assert sel(m * n - 1, m, n) == -11                 # the last batch runs into the next column
    assert sel(m, m * p, n) >= 0 and sel(m, m * p - 1, n) == -12      # packed batches, one element short
    assert sel(m, 0, 1) >= 0                           # one batch: its stride does not matter
    assert sel(m, 0, 2) == -12
