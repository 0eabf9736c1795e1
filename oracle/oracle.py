"""numpy front end of the CPU oracle (oracle/contract_oracle.c).

TEST INFRASTRUCTURE ONLY.  The oracle is the plain definition the GPU library is
checked against: eq. (1) of section II-B evaluated as nested loops over
column-major strided tensors (section III-B), and the loop-of-GEMMs definition
of StridedBatchedGemm (Listing 1, section III-D).  It shares no code with the GPU
library; only tests/, the smoke check and the benchmark's cpu_baseline leg may
import it.

All values travel as fp64 (fp32 and bf16 inputs are exact in fp64); `wide=True`
accumulates in long double.
"""
import ctypes
import os

import numpy as np

try:                                    # imported as package module (tests, bench)
    from . import build as _build
except ImportError:                     # run as a loose script
    import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build.build())
        i64p = ctypes.POINTER(ctypes.c_int64)
        f64p = ctypes.POINTER(ctypes.c_double)
        tensor = [ctypes.c_char_p, i64p, i64p, f64p]
        lib.oracle_contract.restype = ctypes.c_int
        lib.oracle_contract.argtypes = tensor * 3 + [ctypes.c_double, ctypes.c_double, ctypes.c_int]
        lib.oracle_contract_at.restype = ctypes.c_int
        lib.oracle_contract_at.argtypes = tensor * 3 + [ctypes.c_double, ctypes.c_double, ctypes.c_int,
                                                        ctypes.c_int64, i64p, f64p]
        lib.oracle_sb_gemm.restype = ctypes.c_int
        lib.oracle_sb_gemm.argtypes = ([ctypes.c_char, ctypes.c_char] + [ctypes.c_int64] * 3 +
                                       [ctypes.c_double, f64p, ctypes.c_int64, ctypes.c_int64,
                                        f64p, ctypes.c_int64, ctypes.c_int64,
                                        ctypes.c_double, f64p, ctypes.c_int64, ctypes.c_int64,
                                        ctypes.c_int64, ctypes.c_int])
        _lib = lib
    return _lib


def _i64(seq):
    arr = np.ascontiguousarray(np.asarray(list(seq), dtype=np.int64))
    if arr.size == 0:
        arr = np.zeros(1, dtype=np.int64)
    return arr


def _p(arr, ctype):
    return arr.ctypes.data_as(ctypes.POINTER(ctype))


def packed_ld(dims):
    """Packed column-major strides: ld<0> = 1, ld<i> = prod_{j<i} dim<j> (section III-B)."""
    ld, acc = [], 1
    for d in dims:
        ld.append(acc)
        acc *= int(d)
    return ld


def _span(dims, ld):
    """Number of buffer elements a strided tensor touches (0 if it is empty)."""
    if any(int(d) == 0 for d in dims):
        return 0
    return 1 + sum((int(d) - 1) * int(s) for d, s in zip(dims, ld))


def contract_strided(modesA, dimsA, ldA, bufA, modesB, dimsB, ldB, bufB,
                     modesC, dimsC, ldC, bufC, alpha=1.0, beta=0.0, wide=True):
    """eq. (1) on flat fp64 buffers with explicit per-mode strides; returns a new C buffer."""
    lib = _load()
    a = np.ascontiguousarray(bufA, dtype=np.float64).ravel()
    b = np.ascontiguousarray(bufB, dtype=np.float64).ravel()
    c = np.array(bufC, dtype=np.float64, copy=True).ravel()
    for buf, dims, ld, name in ((a, dimsA, ldA, "A"), (b, dimsB, ldB, "B"), (c, dimsC, ldC, "C")):
        if any(int(s) < 0 for s in ld) or _span(dims, ld) > max(buf.size, 0):
            raise ValueError("tensor %s does not fit its buffer" % name)
    dA, lA, dB, lB, dC, lC = map(_i64, (dimsA, ldA, dimsB, ldB, dimsC, ldC))
    if a.size == 0: a = np.zeros(1)
    if b.size == 0: b = np.zeros(1)
    cc = c if c.size else np.zeros(1)
    rc = lib.oracle_contract(modesA.encode(), _p(dA, ctypes.c_int64), _p(lA, ctypes.c_int64), _p(a, ctypes.c_double),
                             modesB.encode(), _p(dB, ctypes.c_int64), _p(lB, ctypes.c_int64), _p(b, ctypes.c_double),
                             modesC.encode(), _p(dC, ctypes.c_int64), _p(lC, ctypes.c_int64), _p(cc, ctypes.c_double),
                             float(alpha), float(beta), int(bool(wide)))
    if rc != 0:
        raise ValueError("oracle_contract rejected its arguments (code %d)" % rc)
    return c


def _dims_of(modesA, A, modesB, B, modesC):
    if A.ndim != len(modesA) or B.ndim != len(modesB):
        raise ValueError("array order does not match its mode string")
    ext = {}
    for modes, X in ((modesA, A), (modesB, B)):
        for ch, d in zip(modes, X.shape):
            if ext.setdefault(ch, int(d)) != int(d):
                raise ValueError("index %r has two different extents" % ch)
    try:
        return [ext[ch] for ch in modesC]
    except KeyError as e:
        raise ValueError("index %s of C is in neither A nor B" % e)


def contract(modesA, A, modesB, B, modesC, C=None, alpha=1.0, beta=0.0, wide=True):
    """C_modesC = alpha * A_modesA * B_modesB + beta * C_modesC for numpy arrays of logical shape.

    Returns a new Fortran-ordered fp64 array.  `C` (the old value) is needed only when beta != 0.
    """
    A = np.asarray(A)
    B = np.asarray(B)
    dimsC = _dims_of(modesA, A, modesB, B, modesC)
    a = np.array(A, dtype=np.float64, order="F")
    b = np.array(B, dtype=np.float64, order="F")
    if C is None:
        if beta != 0.0:
            raise ValueError("beta != 0 needs the old C")
        c = np.zeros(dimsC, dtype=np.float64, order="F")
    else:
        c = np.array(C, dtype=np.float64, order="F")
        if list(c.shape) != dimsC:
            raise ValueError("C has the wrong shape")
    out = contract_strided(modesA, a.shape, packed_ld(a.shape), a.ravel(order="F"),
                           modesB, b.shape, packed_ld(b.shape), b.ravel(order="F"),
                           modesC, dimsC, packed_ld(dimsC), c.ravel(order="F"),
                           alpha, beta, wide)
    return out.reshape(dimsC, order="F")


def contract_at(modesA, A, modesB, B, modesC, cidx, C=None, alpha=1.0, beta=0.0, wide=True):
    """Values of eq. (1) at the output multi-indices `cidx` (shape [nsamples, order(C)]) only."""
    lib = _load()
    A = np.asarray(A)
    B = np.asarray(B)
    dimsC = _dims_of(modesA, A, modesB, B, modesC)
    a = np.array(A, dtype=np.float64, order="F")
    b = np.array(B, dtype=np.float64, order="F")
    if C is None:
        if beta != 0.0:
            raise ValueError("beta != 0 needs the old C")
        c = np.zeros(1, dtype=np.float64)
        ldC = [0] * len(dimsC)
    else:
        c = np.array(C, dtype=np.float64, order="F")
        ldC = packed_ld(dimsC)
    idx = np.ascontiguousarray(np.asarray(cidx, dtype=np.int64).reshape(-1, max(len(dimsC), 1)))
    ns = idx.shape[0] if len(dimsC) else 1
    out = np.zeros(max(ns, 1), dtype=np.float64)
    af, bf, cf = a.ravel(order="F"), b.ravel(order="F"), c.ravel(order="F")
    if af.size == 0: af = np.zeros(1)
    if bf.size == 0: bf = np.zeros(1)
    dA, lA = _i64(a.shape), _i64(packed_ld(a.shape))
    dB, lB = _i64(b.shape), _i64(packed_ld(b.shape))
    dC, lC = _i64(dimsC), _i64(ldC)
    rc = lib.oracle_contract_at(modesA.encode(), _p(dA, ctypes.c_int64), _p(lA, ctypes.c_int64), _p(af, ctypes.c_double),
                                modesB.encode(), _p(dB, ctypes.c_int64), _p(lB, ctypes.c_int64), _p(bf, ctypes.c_double),
                                modesC.encode(), _p(dC, ctypes.c_int64), _p(lC, ctypes.c_int64), _p(cf, ctypes.c_double),
                                float(alpha), float(beta), int(bool(wide)),
                                ns, _p(idx, ctypes.c_int64), _p(out, ctypes.c_double))
    if rc != 0:
        raise ValueError("oracle_contract_at rejected its arguments (code %d)" % rc)
    return out[:ns]


def sb_gemm(opA, opB, m, n, k, alpha, A, lda, loa, B, ldb, lob, beta, C, ldc, loc, batch, wide=True):
    """Listing 1 on flat fp64 buffers (element offsets); returns a new C buffer."""
    lib = _load()
    a = np.ascontiguousarray(A, dtype=np.float64).ravel()
    b = np.ascontiguousarray(B, dtype=np.float64).ravel()
    c = np.array(C, dtype=np.float64, copy=True).ravel()

    def need(op, rows, cols, ld, lo):       # stored matrix is rows x cols before op
        r, cdim = (rows, cols) if op == "N" else (cols, rows)
        if r == 0 or cdim == 0 or batch == 0:
            return 0
        return (batch - 1) * lo + (cdim - 1) * ld + r

    if min(lda, loa, ldb, lob, ldc, loc) < 0:
        raise ValueError("negative stride")
    if need(opA, m, k, lda, loa) > a.size or need(opB, k, n, ldb, lob) > b.size \
            or need("N", m, n, ldc, loc) > c.size:
        raise ValueError("operand does not fit its buffer")
    if a.size == 0: a = np.zeros(1)
    if b.size == 0: b = np.zeros(1)
    cc = c if c.size else np.zeros(1)
    rc = lib.oracle_sb_gemm(opA.encode(), opB.encode(), m, n, k, float(alpha),
                            _p(a, ctypes.c_double), lda, loa, _p(b, ctypes.c_double), ldb, lob,
                            float(beta), _p(cc, ctypes.c_double), ldc, loc, batch, int(bool(wide)))
    if rc != 0:
        raise ValueError("oracle_sb_gemm rejected its arguments (code %d)" % rc)
    return c
