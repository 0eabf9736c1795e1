"""The comparison gates the GPU tests use (helpers.assert_close) checked on the CPU: honest
fp32 / bf16 arithmetic passes, and mistakes planted in a copy of the oracle's result -- one dropped
term in one element, two swapped neighbours, one stale tile -- are caught although the relative
Frobenius error alone would let them through."""
import numpy as np
import pytest

from helpers import TOL, assert_close, elementwise_bound, gemm_window_mask, rel_fro
from oracle import oracle
from paper_1606_05696_amd import inputs


def _case(dtype, m=96, n=80, p=7, k=128, seed=5):
    A = inputs.make_tensor(seed, [m, k], dtype)
    B = inputs.make_tensor(seed + 1, [k, n, p], dtype)
    ref = oracle.contract("mk", A, "knp", B, "mnp", wide=(dtype == "f64"))
    return A, B, ref


def _device_like(A, B, dtype):
    """The same sums in the accumulation type of the device path (another summation order)."""
    acc = np.float64 if dtype == "f64" else np.float32
    out = np.einsum("mk,knp->mnp", A.astype(acc), B.astype(acc), optimize=True).astype(acc)
    if dtype == "bf16":
        out = inputs.round_to_bf16(out)
    return out.astype(np.float64)


@pytest.mark.parametrize("dtype", ["f64", "f32", "bf16"])
def test_honest_arithmetic_passes(dtype):
    A, B, ref = _case(dtype)
    got = _device_like(A, B, dtype)
    err = assert_close(got, ref, dtype, 128, np.abs(A).max(), np.abs(B).max())
    assert err <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f64", "f32", "bf16"])
def test_planted_mistakes_are_caught(dtype):
    A, B, ref = _case(dtype)
    good = _device_like(A, B, dtype)
    amax, bmax = np.abs(A).max(), np.abs(B).max()

    def fails(bad):
        with pytest.raises(AssertionError):
            assert_close(bad, ref, dtype, 128, amax, bmax)

    # one term of one sum dropped (the largest of that sum, as an index off by one at an edge would)
    dropped = good.copy()
    terms = A[3, :].astype(np.float64) * B[:, 5, 2].astype(np.float64)
    dropped[3, 5, 2] -= terms[np.argmax(np.abs(terms))]
    fails(dropped)
    # two neighbouring outputs swapped
    swapped = good.copy()
    swapped[10, 7, 1], swapped[11, 7, 1] = good[11, 7, 1], good[10, 7, 1]
    fails(swapped)
    # a 16 x 16 block never written (stale zeros)
    stale = good.copy()
    stale[32:48, 32:48, 4] = 0.0
    fails(stale)
    if dtype == "bf16":
        # ... and at this tolerance the Frobenius gate alone would have accepted the first two
        assert rel_fro(dropped, ref) <= TOL[dtype] and rel_fro(swapped, ref) <= TOL[dtype]


def test_bound_scales_with_the_arithmetic():
    ref = np.array([0.0, 1.0, -100.0])
    b32 = elementwise_bound(ref, "f32", 512, 1.0, 1.0)
    b64 = elementwise_bound(ref, "f64", 512, 1.0, 1.0)
    bb = elementwise_bound(ref, "bf16", 512, 1.0, 1.0)
    assert np.allclose(b32, 516 * 2.0 ** -24 * 512) and np.allclose(b64, 516 * 2.0 ** -53 * 512)
    assert np.all(bb >= b32) and np.isclose(bb[2] - bb[0], 100 * 2.0 ** -8)
    # alpha = 0, beta = 0.5: only the old C matters
    c_old = np.array([2.0, 0.0, -4.0])
    assert np.allclose(elementwise_bound(ref, "f32", 0, 1.0, 1.0, 0.0, 0.5, c_old), 4 * 2.0 ** -24 * 0.5 * np.abs(c_old))


def test_window_mask():
    mask = gemm_window_mask(200, 3, 4, 5, 30, 6)
    assert mask.sum() == 3 * 4 * 6
    assert mask[0] and mask[2] and not mask[3] and mask[5] and mask[30 * 5 + 3 * 5 + 2] and not mask[199]
    assert gemm_window_mask(10, 0, 4, 5, 30, 6).sum() == 0
