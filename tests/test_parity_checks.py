"""The float comparison rules of the GPU parity tests, tried on the CPU with planted mistakes: an answer
that is wrong only deep inside a long segment must be rejected (there the gate relative to the running sum
of |x| allows more than the result's own size)."""
import numpy as np
import pytest

import oracle
from parity_util import check_scan, check_sum


def _alternating(n):
    x = np.ones(n, dtype=np.float32)
    x[1::2] = -1.0                       # running sum 1, 0, 1, 0, ...: |ref| <= 1 while A_i = i + 1
    f = np.zeros(n, dtype=np.uint8)
    f[0] = 1
    return x, f


def test_correct_answer_passes():
    x, f = _alternating(1 << 20)
    good = oracle.segscan(x, f).astype(np.float32)
    assert check_scan(good, x, f) == 0.0
    assert check_sum(np.array([0.0], dtype=np.float32), 1, x, f) == 0.0


@pytest.mark.parametrize("mistake", ["zeros in the tail", "shifted by one", "carry dropped at a tile border"])
def test_wrong_answer_deep_inside_a_long_segment_is_rejected(mistake):
    n = 1 << 20
    x, f = _alternating(n)
    bad = oracle.segscan(x, f).astype(np.float32)
    if mistake == "zeros in the tail":
        bad[n // 2:] = 0.0
    elif mistake == "shifted by one":
        bad[n // 2:] = bad[n // 2 - 1:-1]
    else:
        bad[n // 2 + 1:] -= 1.0          # as if the carry into position n/2+1 had been lost
    # the gate alone would let all of these through: |err| <= 1 against 1e-4 * A_i > 50 there
    A = np.arange(1, n + 1, dtype=np.float64)
    err = np.abs(bad.astype(np.float64) - oracle.segscan(x, f))
    assert (err <= 1e-4 * np.maximum(A, 1.0)).all() and err.max() == 1.0
    with pytest.raises(AssertionError):
        check_scan(bad, x, f)


def test_wrong_sum_of_a_long_segment_is_rejected():
    x, f = _alternating((1 << 20) + 1)   # the sum is 1
    with pytest.raises(AssertionError):
        check_sum(np.array([0.0], dtype=np.float32), 1, x, f)
    with pytest.raises(AssertionError):
        check_sum(np.array([2.0], dtype=np.float32), 1, x, f)
    assert check_sum(np.array([1.0], dtype=np.float32), 1, x, f) == 0.0


def test_nan_is_rejected():
    x, f = _alternating(4096)
    bad = oracle.segscan(x, f).astype(np.float32)
    bad[100] = np.nan
    with pytest.raises(AssertionError):
        check_scan(bad, x, f)
