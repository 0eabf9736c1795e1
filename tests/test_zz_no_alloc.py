"""sb_sym_eig_static, the entry point for callers that cannot allocate: its workspace is a device
array inside the library.  Checked against sb_sym_eig (caller's workspace, same kernels) on two
calls in a row, the second on a smaller matrix, so that what the first call left in the shared
array is seen not to matter."""
import numpy as np
import pytest

import paper_1606_05696_amd as sb
from helpers import from_dev, to_dev
from paper_1606_05696_amd import inputs

pytestmark = pytest.mark.gpu

NP_DTYPE = {"f64": np.float64, "f32": np.float32}


def gram(seed, n, dtype):
    X = inputs.uniform_tensor(seed, [2 * n + 3, n])
    X = X * (1.0 / (1.0 + np.arange(n)))
    return (X.T @ X).astype(NP_DTYPE[dtype]).astype(np.float64)


def solve(dtype, S, n, static):
    import torch
    tS = to_dev(S, dtype)
    tV = to_dev(np.full((n, n), np.nan), dtype)
    tl = to_dev(np.full(n, np.nan), dtype)
    if static:
        sb.sb_sym_eig_static(n, tS, tV, tl, dt=dtype)
    else:
        nbytes = sb.sb_sym_eig_workspace(dtype, n)[1]
        ws = torch.empty((nbytes + 255) // 256 * 256, dtype=torch.uint8, device="cuda")
        sb.sb_sym_eig(n, tS, tV, tl, ws, dt=dtype)
    torch.cuda.synchronize()
    return from_dev(tl), from_dev(tV, [n, n])


@pytest.mark.parametrize("dtype", ["f64", "f32"])
def test_static_workspace_entry_matches_the_workspace_entry(dtype):
    # first the largest order it takes (multi-launch path: every block of the array is used), then a
    # smaller one on the same stream (in-LDS path), then the large one again
    for step, n in enumerate((sb.SB_SYM_EIG_STATIC_MAX_N, 96, 150)):
        S = gram(900 + step, n, dtype)
        w_ref, V_ref = solve(dtype, S, n, static=False)
        w, V = solve(dtype, S, n, static=True)
        assert np.isfinite(w).all() and np.isfinite(V).all()
        # same kernels, same order of operations: the results agree to the last bit; the tolerance
        # asked of any fp64 / fp32 result would be 1e-12 / 1e-5 relative
        tol = 1e-12 if dtype == "f64" else 1e-5
        assert np.linalg.norm(w - w_ref) <= tol * np.linalg.norm(w_ref), (n, step)
        assert np.linalg.norm(V - V_ref) <= tol * np.linalg.norm(V_ref), (n, step)
        assert np.array_equal(w, w_ref) and np.array_equal(V, V_ref), (n, step)
        # and it is an eigen-decomposition
        eps = 1e-13 if dtype == "f64" else 2e-5
        assert np.max(np.abs(S @ V - V * w)) <= eps * w[0] * max(n, 8)


def test_static_workspace_entry_rejects_larger_orders():
    import torch
    n = sb.SB_SYM_EIG_STATIC_MAX_N + 1
    t = torch.zeros(n * n, dtype=torch.float32, device="cuda")
    assert sb.sb_sym_eig_static(n, t, t, t, dt="f32", check=False) == -2
    assert sb.sb_sym_eig_static(0, t, t, t, dt="f32", check=False) == -2
    assert sb.sb_sym_eig_static(4, t, t, t, dt="bf16", check=False) == -1
    assert sb.sb_sym_eig_static(4, None, t, t, dt="f32", check=False) == -3
