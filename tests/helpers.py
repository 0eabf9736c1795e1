"""Helpers shared by the test modules (host side only)."""
import itertools
import re

import numpy as np

OPS_PLAIN = (0, 1)


def cases_2x3():
    """(modesA, modesB) of the 36 order-2 x order-3 single-mode contractions into C_mnp."""
    out = []
    for free_a in "mnp":
        rest = [c for c in "mnp" if c != free_a]
        for ma in (free_a + "k", "k" + free_a):
            for perm in itertools.permutations(["k"] + rest):
                out.append((ma, "".join(perm)))
    return out


def cases_general(order_a, order_b):
    """All single-mode contractions between tensors of the given orders with C in canonical order."""
    free = "mnpqrs"[:order_a + order_b - 2]
    out = []
    for perm in itertools.permutations(free):
        fa, fb = perm[:order_a - 1], perm[order_a - 1:]
        for ia in range(order_a):
            for ib in range(order_b):
                ma = "".join(fa[:ia]) + "k" + "".join(fa[ia:])
                mb = "".join(fb[:ib]) + "k" + "".join(fb[ib:])
                out.append((ma, mb, free))
    return out


def split_kernel(text):
    """'C_mn[p] = B_km[p]^T A_nk^T' -> dict(A='nk', B='km[p]', C='mn[p]') (annotated mode strings)."""
    lhs, rhs = text.split("=")
    out = {"C": lhs.strip()[2:]}
    for term in rhs.split():
        out[term[0]] = term[2:].replace("^T", "")
    return out


def strip_annotations(s):
    return re.sub(r"[\[\]\(\)]", "", s)


def packed(dims):
    ld, acc = [], 1
    for d in dims:
        ld.append(acc)
        acc *= int(d)
    return ld


def run_plan_numpy(plan, A, B, C0, alpha, beta):
    """Execute an sb_plan with numpy on flat column-major buffers: a loop of small matrix products.

    Independent of the GPU kernels: it only follows the meaning of the plan's fields
    (sbgemm.h: sb_plan, sb_op).  Returns the new flat C buffer (fp64).
    """
    L, R = (B, A) if plan.left_is_B else (A, B)
    L = np.asarray(L, dtype=np.float64)
    R = np.asarray(R, dtype=np.float64)
    C = np.array(C0, dtype=np.float64, copy=True)
    m, n, k = plan.m, plan.n, plan.k

    def strides(op, ld, ex):      # (row stride, col stride) of op(X)
        return {0: (1, ld), 1: (ld, 1), 2: (ld, ex), 3: (ex, ld)}[op]

    rsL, csL = strides(plan.opL, plan.ldL, plan.exL)
    rsR, csR = strides(plan.opR, plan.ldR, plan.exR)
    nb = plan.nbatch
    for idx in itertools.product(*[range(plan.batch[q]) for q in range(nb)]):
        oL = sum(i * plan.strideL[q] for q, i in enumerate(idx))
        oR = sum(i * plan.strideR[q] for q, i in enumerate(idx))
        oC = sum(i * plan.strideC[q] for q, i in enumerate(idx))
        Lm = np.array([[L[oL + i * rsL + l * csL] for l in range(k)] for i in range(m)]).reshape(m, k)
        Rm = np.array([[R[oR + l * rsR + j * csR] for j in range(n)] for l in range(k)]).reshape(k, n)
        P = alpha * (Lm @ Rm)
        for j in range(n):
            for i in range(m):
                o = oC + i + j * plan.ldC
                C[o] = P[i, j] + (beta * C[o] if beta != 0 else 0.0)
    return C


# ------------------------------------------------------------------ device helpers (GPU tests)

TOL = {"f64": 1e-12, "f32": 1e-5, "bf16": 2e-2}      # relative Frobenius error allowed per element type


def to_dev(x, dtype):
    """Column-major flat device buffer holding the values of numpy array `x` (any shape)."""
    import torch
    from paper_1606_05696_amd import inputs
    flat = np.ascontiguousarray(np.asarray(x).ravel(order="F"))
    if dtype == "f64":
        return torch.from_numpy(flat.astype(np.float64)).cuda()
    if dtype == "f32":
        return torch.from_numpy(flat.astype(np.float32)).cuda()
    bits = inputs.bf16_bits(inputs.round_to_bf16(flat.astype(np.float32)))
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def from_dev(t, shape=None):
    """fp64 numpy values of a flat device buffer, optionally reshaped column-major."""
    import torch
    out = t.detach().to(torch.float64).cpu().numpy()
    return out if shape is None else out.reshape(shape, order="F")


def quantise(x, dtype):
    """The values the device will actually hold for host values `x`."""
    from paper_1606_05696_amd import inputs
    x = np.asarray(x)
    if dtype == "f64":
        return x.astype(np.float64)
    if dtype == "f32":
        return x.astype(np.float32).astype(np.float64)
    return inputs.round_to_bf16(x.astype(np.float32)).astype(np.float64)


def rel_fro(got, ref):
    got = np.asarray(got, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    den = np.linalg.norm(ref)
    return np.linalg.norm(got - ref) / den if den > 0 else np.linalg.norm(got)


# Element-wise bound.  A relative Frobenius norm over millions of outputs lets a handful of wrong
# elements through (at bf16's 2e-2 even a whole wrong tile), so every comparison also bounds each
# element by what the arithmetic can do.  The device computes v = alpha * sum_k a b + beta * c in the
# accumulation type (unit roundoff u: 2^-24 for f32 and bf16, 2^-53 for f64) in some order, then
# stores it (bf16: one more rounding to nearest even, relative 2^-8: 8 significant bits).  Any order of K products, K
# additions and the alpha / beta arithmetic obeys the standard running-error bound
#     |v - exact| <= (K + 4) u (|alpha| sum_k |a||b| + |beta||c|)  <=  (K + 4) u (|alpha| K amax bmax + |beta||c|),
# and |stored - v| <= u_out |v|.  The reference is exact to 2^-53 or better, which the bound absorbs.
ACC_UNIT = {"f64": 2.0 ** -53, "f32": 2.0 ** -24, "bf16": 2.0 ** -24}
OUT_UNIT = {"f64": 0.0, "f32": 0.0, "bf16": 2.0 ** -8}


def elementwise_bound(ref, dtype, K, amax, bmax, alpha=1.0, beta=0.0, c_old=None):
    """Largest |got - ref| the arithmetic allows, per element of `ref` (an array of its shape)."""
    ref = np.asarray(ref, dtype=np.float64)
    mag = abs(alpha) * max(K, 0) * float(amax) * float(bmax) * np.ones_like(ref)
    if beta != 0.0 and c_old is not None:
        mag = mag + abs(beta) * np.abs(np.asarray(c_old, dtype=np.float64).reshape(ref.shape))
    acc = (max(K, 0) + 4) * ACC_UNIT[dtype] * mag
    return OUT_UNIT[dtype] * (np.abs(ref) + acc) + acc


def assert_close(got, ref, dtype, K, amax, bmax, alpha=1.0, beta=0.0, c_old=None, what=""):
    """The two gates of every GPU comparison: relative Frobenius error within TOL[dtype] and every
    element within elementwise_bound().  Returns the relative Frobenius error."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), ("non-finite output", what)
    err = rel_fro(got, ref)
    assert err <= TOL[dtype], ("relative Frobenius error", err, what)
    excess = np.abs(got - ref) - elementwise_bound(ref, dtype, K, amax, bmax, alpha, beta, c_old)
    if excess.size and excess.max() > 0:
        at = np.unravel_index(int(np.argmax(excess)), excess.shape)
        raise AssertionError("element %s: got %r, reference %r, %d elements beyond the element-wise bound (%s)"
                             % (at, got[at], ref[at], int((excess > 0).sum()), what))
    return err


def gemm_window_mask(size, m, n, ldc, loc, batch):
    """Boolean mask over a flat C buffer: True where one of the batch's m x n windows lies."""
    mask = np.zeros(size, dtype=bool)
    if m and n and batch:
        i = np.arange(m, dtype=np.int64)[:, None, None]
        j = np.arange(n, dtype=np.int64)[None, :, None]
        p = np.arange(batch, dtype=np.int64)[None, None, :]
        mask[(i + j * ldc + p * loc).ravel()] = True
    return mask
