"""ctypes binding of libsbgemm.so: the same entry points as include/sbgemm.h and include/sbtucker.h,
same names.

Only argument marshalling happens here; every step of the path (planning, kernel selection,
kernels) runs inside the library.  torch is used for device memory and streams only.  There is
no fallback: if the library has not been built, every call raises.
"""
import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libsbgemm.so")

SB_OP_N, SB_OP_T, SB_OP_EX_N, SB_OP_EX_T = 0, 1, 2, 3
SB_F64, SB_F32, SB_BF16 = 0, 1, 2
SB_AUTO, SB_FLATTEN, SB_BATCH_LAST, SB_BATCH_MID, SB_NESTED, SB_LEVEL2 = 0, 1, 2, 3, 4, 5
SB_OK = 0
SB_ERR_MODES, SB_ERR_CONTRACTION, SB_ERR_EXTENT, SB_ERR_STRIDE, SB_ERR_ILLEGAL_EVAL, SB_ERR_NO_DEVICE_CODE = 1, 2, 3, 4, 5, 6
SB_ERR_LAUNCH = 1000
SB_KERNEL_AUTO, SB_KERNEL_GENERIC, SB_KERNEL_TINY, SB_KERNEL_MFMA, SB_KERNEL_THIN, SB_KERNEL_PANEL = -1, 0, 1, 2, 3, 4
SB_MEMBER_PANEL_4X4, SB_MEMBER_PANEL_WIDE, SB_MEMBER_TINY_WHOLE, SB_MEMBER_TINY_BLOCKS = 1, 2, 1, 2
SB_MEMBER_MFMA_EX_BRICK, SB_MEMBER_MFMA_EX_SMALL, SB_MEMBER_MFMA_EX_DMA = 1, 2, 3
SB_MAX_MODES = 8
SB_MAX_BATCH_LEVELS = 8

OPS = {"N": SB_OP_N, "T": SB_OP_T, "EX_N": SB_OP_EX_N, "EX_T": SB_OP_EX_T}
DTYPES = {"f64": SB_F64, "f32": SB_F32, "bf16": SB_BF16}
STRATEGIES = {"auto": SB_AUTO, "flatten": SB_FLATTEN, "batch_last": SB_BATCH_LAST,
              "batch_mid": SB_BATCH_MID, "nested": SB_NESTED, "level2": SB_LEVEL2}


__all__ = [n for n in dir() if n.startswith("SB_")] + ["SB_SYM_EIG_STATIC_MAX_N"] + [
    "OPS", "DTYPES", "STRATEGIES", "sb_plan", "SbError", "load", "sb_status_string", "sb_gemm", "sb_gemm2", "sb_gemm_nested",
    "sb_contract_plan", "sb_contract", "sb_plan_launch", "sb_plan_launches", "sb_force_kernel", "sb_last_kernel", "sb_last_kernel_member",
    "sb_select_kernel", "sb_plan_cache_enable", "sb_permute", "sb_tucker_workspace", "sb_tucker_hooi", "sb_sym_eig_workspace", "sb_sym_eig", "sb_sym_eig_static",
    "sb_probe_mfma"]


class sb_plan(ctypes.Structure):
    _fields_ = [("nbatch", ctypes.c_int32), ("exceptional", ctypes.c_int32), ("left_is_B", ctypes.c_int32),
                ("opL", ctypes.c_int32), ("opR", ctypes.c_int32),
                ("m", ctypes.c_int64), ("n", ctypes.c_int64), ("k", ctypes.c_int64),
                ("ldL", ctypes.c_int64), ("ldR", ctypes.c_int64), ("ldC", ctypes.c_int64),
                ("exL", ctypes.c_int64), ("exR", ctypes.c_int64),
                ("batch", ctypes.c_int64 * SB_MAX_BATCH_LEVELS),
                ("strideL", ctypes.c_int64 * SB_MAX_BATCH_LEVELS),
                ("strideR", ctypes.c_int64 * SB_MAX_BATCH_LEVELS),
                ("strideC", ctypes.c_int64 * SB_MAX_BATCH_LEVELS),
                ("notation", ctypes.c_char * 192)]

    def text(self):
        return self.notation.decode()


class SbError(RuntimeError):
    def __init__(self, fn, status):
        self.status = status
        super().__init__("%s failed with status %d: %s" % (fn, status, sb_status_string(status)))


_lib = None


def load():
    """Load libsbgemm.so (once).  Raises if it has not been built: there is no other path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libsbgemm.so is missing at %s; build it with "
                           "`python -m paper_1606_05696_amd.build` (needs hipcc)" % LIB_PATH)
    import torch  # noqa: F401  (loads the HIP runtime that owns torch's device memory first)
    lib = ctypes.CDLL(LIB_PATH)
    i64, dbl, vp, cp = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p, ctypes.c_char_p
    i64p = ctypes.POINTER(ctypes.c_int64)
    ci = ctypes.c_int
    lib.sb_gemm.restype = ci
    lib.sb_gemm.argtypes = [ci, ci, ci, i64, i64, i64, dbl, vp, i64, i64, vp, i64, i64, dbl, vp, i64, i64, i64, vp]
    lib.sb_gemm2.restype = ci
    lib.sb_gemm2.argtypes = [ci, ci, ci, i64, i64, i64, dbl, vp, i64, i64, i64, vp, i64, i64, i64,
                             dbl, vp, i64, i64, i64, i64, i64, vp]
    lib.sb_gemm_nested.restype = ci
    lib.sb_gemm_nested.argtypes = [ci, ci, ci, i64, i64, i64, dbl, vp, i64, i64p, vp, i64, i64p, dbl, vp, i64, i64p, ci, i64p, vp]
    lib.sb_contract_plan.restype = ci
    lib.sb_contract_plan.argtypes = [cp, cp, cp, i64p, i64p, i64p, i64p, i64p, i64p, ci, ctypes.POINTER(sb_plan)]
    lib.sb_contract.restype = ci
    lib.sb_contract.argtypes = [ci, cp, cp, cp, dbl, vp, i64p, i64p, vp, i64p, i64p, dbl, vp, i64p, i64p, ci, vp]
    lib.sb_plan_launch.restype = ci
    lib.sb_plan_launch.argtypes = [ci, ctypes.POINTER(sb_plan), dbl, vp, vp, dbl, vp, vp]
    lib.sb_plan_launches.restype = i64
    lib.sb_plan_launches.argtypes = [ctypes.POINTER(sb_plan)]
    lib.sb_status_string.restype = cp
    lib.sb_status_string.argtypes = [ci]
    lib.sb_force_kernel.restype = ci
    lib.sb_force_kernel.argtypes = [ci]
    lib.sb_permute.restype = ci
    lib.sb_permute.argtypes = [ci, ci, i64p, ctypes.POINTER(ci), vp, vp, vp]
    lib.sb_plan_cache_enable.restype = ci
    lib.sb_plan_cache_enable.argtypes = [ci]
    lib.sb_last_kernel.restype = ci
    lib.sb_last_kernel.argtypes = []
    lib.sb_last_kernel_member.restype = ci
    lib.sb_last_kernel_member.argtypes = []
    lib.sb_select_kernel.restype = ci
    lib.sb_select_kernel.argtypes = [ci, ci, ci, i64, i64, i64, i64, i64, i64, i64, i64, i64, i64]
    lib.sb_probe_mfma.restype = ci
    lib.sb_probe_mfma.argtypes = [ci, ci, vp, i64, vp, ctypes.POINTER(dbl)]
    lib.sb_tucker_workspace.restype = ci
    lib.sb_tucker_workspace.argtypes = [ci, i64, i64, i64, i64, i64, i64, ci, i64p]
    lib.sb_tucker_hooi.restype = ci
    lib.sb_tucker_hooi.argtypes = [ci, vp, i64, i64, i64, i64, i64, i64, ci, ci, vp, vp, vp, vp, vp, i64, vp]
    lib.sb_sym_eig_workspace.restype = ci
    lib.sb_sym_eig_workspace.argtypes = [ci, i64, i64p]
    lib.sb_sym_eig.restype = ci
    lib.sb_sym_eig.argtypes = [ci, i64, vp, vp, vp, ci, vp, i64, vp]
    lib.sb_sym_eig_static.restype = ci
    lib.sb_sym_eig_static.argtypes = [ci, i64, vp, vp, vp, ci, vp]
    _lib = lib
    return lib


def _ptr(x):
    """Device pointer of a torch tensor, or an integer address passed through."""
    if x is None:
        return None
    if x.__class__ is int:
        return x
    return x.data_ptr()


_TORCH_DTYPES = None


def _dtype_of(dt, *tensors):
    global _TORCH_DTYPES
    if dt is not None:
        return DTYPES[dt] if dt.__class__ is str else dt
    if _TORCH_DTYPES is None:
        import torch
        _TORCH_DTYPES = {torch.float64: SB_F64, torch.float32: SB_F32, torch.bfloat16: SB_BF16}
    kind = None
    for t in tensors:
        d = getattr(t, "dtype", None)
        if d is None:
            continue
        if kind is None:
            kind = d
        elif d is not kind:
            raise TypeError("the tensors have different element types; pass dt")
    if kind is None or kind not in _TORCH_DTYPES:
        raise TypeError("cannot infer the element type from the tensors; pass dt")
    return _TORCH_DTYPES[kind]


_RAW_STREAM = None


def _stream(stream, ref=None):
    """hipStream_t (as an integer) to launch on: the one given, else torch's current stream of the
    device that holds `ref`.  torch.cuda.current_stream() builds a Stream object (2.6 us); the raw
    getter behind it costs 0.1 us, which matters for contractions that are launch-bound."""
    global _RAW_STREAM
    if stream is None:
        import torch
        if _RAW_STREAM is None:
            _RAW_STREAM = getattr(torch._C, "_cuda_getCurrentRawStream", False)
        if _RAW_STREAM:
            dev = ref.device.index if ref is not None and hasattr(ref, "device") else None
            return _RAW_STREAM(torch.cuda.current_device() if dev is None else dev)
        return torch.cuda.current_stream().cuda_stream
    if stream.__class__ is int:
        return stream
    return stream.cuda_stream


_ARRAYS = {}
_BYTES = {}


def _i64arr(seq):
    """ctypes int64 array for a sequence of extents/strides (cached: calls repeat the same shapes)."""
    if seq is None:
        return None
    key = tuple(seq)
    arr = _ARRAYS.get(key)
    if arr is None:
        vals = [int(v) for v in key]
        arr = (ctypes.c_int64 * max(len(vals), 1))(*vals)
        if len(_ARRAYS) < 4096:
            _ARRAYS[key] = arr
    return arr


def _b(text):
    out = _BYTES.get(text)
    if out is None:
        out = text.encode()
        if len(_BYTES) < 4096:
            _BYTES[text] = out
    return out


def _op(op):
    return OPS[op] if op.__class__ is str else op


def _strat(s):
    return STRATEGIES[s] if s.__class__ is str else s


def sb_status_string(status):
    return load().sb_status_string(int(status)).decode()


def sb_gemm(transA, transB, m, n, k, alpha, A, lda, strideA, B, ldb, strideB, beta, C, ldc, strideC,
            batch, dt=None, stream=None, check=True):
    """C_p = alpha*opA(A_p)*opB(B_p) + beta*C_p over device buffers (see sbgemm.h: sb_gemm)."""
    rc = load().sb_gemm(_dtype_of(dt, A, B, C), _op(transA), _op(transB), m, n, k, float(alpha),
                        _ptr(A), lda, strideA, _ptr(B), ldb, strideB, float(beta), _ptr(C), ldc, strideC,
                        batch, _stream(stream, C))
    if check and rc != SB_OK:
        raise SbError("sb_gemm", rc)
    return rc


def sb_gemm2(transA, transB, m, n, k, alpha, A, lda, strideA0, strideA1, B, ldb, strideB0, strideB1,
             beta, C, ldc, strideC0, strideC1, batch0, batch1, dt=None, stream=None, check=True):
    """Two batch levels in one launch (see sbgemm.h: sb_gemm2)."""
    rc = load().sb_gemm2(_dtype_of(dt, A, B, C), _op(transA), _op(transB), m, n, k, float(alpha),
                         _ptr(A), lda, strideA0, strideA1, _ptr(B), ldb, strideB0, strideB1,
                         float(beta), _ptr(C), ldc, strideC0, strideC1, batch0, batch1, _stream(stream, C))
    if check and rc != SB_OK:
        raise SbError("sb_gemm2", rc)
    return rc


def sb_gemm_nested(transA, transB, m, n, k, alpha, A, lda, strideA, B, ldb, strideB, beta, C, ldc, strideC, batch,
                   dt=None, stream=None, check=True):
    """Any number of batch levels in one launch (see sbgemm.h: sb_gemm_nested); strideX and batch are sequences, level 0 first."""
    rc = load().sb_gemm_nested(_dtype_of(dt, A, B, C), _op(transA), _op(transB), m, n, k, float(alpha),
                               _ptr(A), lda, _i64arr(strideA), _ptr(B), ldb, _i64arr(strideB),
                               float(beta), _ptr(C), ldc, _i64arr(strideC), len(batch), _i64arr(batch), _stream(stream, C))
    if check and rc != SB_OK:
        raise SbError("sb_gemm_nested", rc)
    return rc


def sb_contract_plan(modesA, modesB, modesC, dimsA, dimsB, dimsC=None, stridesA=None, stridesB=None,
                     stridesC=None, strat=SB_AUTO, check=True):
    """Plan a contraction on the host (see sbgemm.h: sb_contract_plan).  Returns (status, sb_plan)."""
    plan = sb_plan()
    rc = load().sb_contract_plan(_b(modesA), _b(modesB), _b(modesC),
                                 _i64arr(dimsA), _i64arr(stridesA), _i64arr(dimsB), _i64arr(stridesB),
                                 _i64arr(dimsC), _i64arr(stridesC), _strat(strat), ctypes.byref(plan))
    if check and rc != SB_OK:
        raise SbError("sb_contract_plan", rc)
    return rc, plan


def sb_contract(modesA, modesB, modesC, alpha, A, dimsA, B, dimsB, beta, C, dimsC=None,
                stridesA=None, stridesB=None, stridesC=None, strat=SB_AUTO, dt=None, stream=None, check=True):
    """C_modesC = alpha*A_modesA*B_modesB + beta*C_modesC on device tensors (see sbgemm.h: sb_contract)."""
    rc = load().sb_contract(_dtype_of(dt, A, B, C), _b(modesA), _b(modesB), _b(modesC),
                            float(alpha), _ptr(A), _i64arr(dimsA), _i64arr(stridesA),
                            _ptr(B), _i64arr(dimsB), _i64arr(stridesB),
                            float(beta), _ptr(C), _i64arr(dimsC), _i64arr(stridesC), _strat(strat), _stream(stream, C))
    if check and rc != SB_OK:
        raise SbError("sb_contract", rc)
    return rc


def sb_plan_launch(plan, alpha, A, B, beta, C, dt=None, stream=None, check=True):
    """Launch a plan made by sb_contract_plan (see sbgemm.h: sb_plan_launch)."""
    rc = load().sb_plan_launch(_dtype_of(dt, A, B, C), ctypes.byref(plan), float(alpha), _ptr(A), _ptr(B),
                               float(beta), _ptr(C), _stream(stream, C))
    if check and rc != SB_OK:
        raise SbError("sb_plan_launch", rc)
    return rc


def sb_force_kernel(kernel_id):
    return load().sb_force_kernel(int(kernel_id))


def sb_last_kernel():
    return load().sb_last_kernel()


def sb_last_kernel_member():
    return load().sb_last_kernel_member()


def sb_permute(dims, perm, src, dst, dt=None, stream=None, check=True):
    """Out-of-place mode permutation of a packed device tensor (see sbgemm.h: sb_permute): dst mode j = src mode perm[j]."""
    order = len(dims)
    d = (ctypes.c_int64 * max(order, 1))(*[int(x) for x in dims])
    p = (ctypes.c_int * max(order, 1))(*[int(x) for x in perm])
    rc = load().sb_permute(_dtype_of(dt, src, dst), order, d, p, _ptr(src), _ptr(dst), _stream(stream, src))
    if check and rc != SB_OK:
        raise SbError("sb_permute", rc)
    return rc


def sb_plan_cache_enable(on):
    return load().sb_plan_cache_enable(int(bool(on)))


def sb_select_kernel(dt, transA, transB, m, n, k, lda, strideA, ldb, strideB, ldc, strideC, batch):
    return load().sb_select_kernel(_dtype_of(dt), _op(transA), _op(transB), m, n, k, lda, strideA, ldb, strideB,
                                   ldc, strideC, batch)


def sb_plan_launches(plan):
    """Number of kernel launches sb_plan_launch issues for this plan (see sbgemm.h)."""
    return load().sb_plan_launches(ctypes.byref(plan))


def sb_probe_mfma(dt, iterations, scratch, stream=None, check=True):
    """Enqueue the pure-MFMA probe kernel (see sbgemm.h: sb_probe_mfma).  Returns (status, flops)."""
    out = dbl_out = ctypes.c_double(0.0)
    rc = load().sb_probe_mfma(_dtype_of(dt), int(iterations), _ptr(scratch), scratch.numel() * scratch.element_size(),
                              _stream(stream), ctypes.byref(out))
    if check and rc != SB_OK:
        raise SbError("sb_probe_mfma", rc)
    return rc, dbl_out.value


def sb_tucker_workspace(dt, m, n, p, i, j, k, with_init=True, check=True):
    """Bytes of device workspace for sb_tucker_hooi (see sbtucker.h).  Returns (status, bytes)."""
    out = ctypes.c_int64(0)
    rc = load().sb_tucker_workspace(_dtype_of(dt), m, n, p, i, j, k, int(bool(with_init)), ctypes.byref(out))
    if check and rc != SB_OK:
        raise SbError("sb_tucker_workspace", rc)
    return rc, out.value


def sb_tucker_hooi(T, dims, core, iterations, A, B, C, G, workspace, init=True, dt=None, stream=None, check=True):
    """Tucker decomposition by HOOI on device tensors (see sbtucker.h: sb_tucker_hooi).  `workspace` is a
    device buffer (torch tensor of any dtype) of at least sb_tucker_workspace(...) bytes."""
    m, n, p = dims
    i, j, k = core
    nbytes = workspace.numel() * workspace.element_size() if hasattr(workspace, "numel") else 0
    rc = load().sb_tucker_hooi(_dtype_of(dt, T, A, B, C, G), _ptr(T), m, n, p, i, j, k, int(iterations), int(bool(init)),
                               _ptr(A), _ptr(B), _ptr(C), _ptr(G), _ptr(workspace), nbytes, _stream(stream, T))
    if check and rc != SB_OK:
        raise SbError("sb_tucker_hooi", rc)
    return rc


def sb_sym_eig_workspace(dt, n, check=True):
    out = ctypes.c_int64(0)
    rc = load().sb_sym_eig_workspace(_dtype_of(dt), n, ctypes.byref(out))
    if check and rc != SB_OK:
        raise SbError("sb_sym_eig_workspace", rc)
    return rc, out.value


def sb_sym_eig(n, S, V, lam, workspace, sweeps=0, dt=None, stream=None, check=True):
    """Eigen-decomposition of a symmetric device matrix by Jacobi rotations (see sbtucker.h: sb_sym_eig)."""
    nbytes = workspace.numel() * workspace.element_size() if hasattr(workspace, "numel") else 0
    rc = load().sb_sym_eig(_dtype_of(dt, S, V, lam), n, _ptr(S), _ptr(V), _ptr(lam), int(sweeps), _ptr(workspace), nbytes,
                           _stream(stream))
    if check and rc != SB_OK:
        raise SbError("sb_sym_eig", rc)
    return rc


SB_SYM_EIG_STATIC_MAX_N = 256


def sb_sym_eig_static(n, S, V, lam, sweeps=0, dt=None, stream=None, check=True):
    """sb_sym_eig with the library's own fixed workspace (see sbtucker.h: sb_sym_eig_static): allocates nothing."""
    rc = load().sb_sym_eig_static(_dtype_of(dt, S, V, lam), n, _ptr(S), _ptr(V), _ptr(lam), int(sweeps), _stream(stream))
    if check and rc != SB_OK:
        raise SbError("sb_sym_eig_static", rc)
    return rc
