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
