"""Pins for the oracle's permutation sigma_(b,N) (Sec. 3.1; Appendix notation item 6)."""
import numpy as np
import pytest

import oracle


def _all_pairs(limit):
    return [(b, N) for N in range(1, limit + 1) for b in range(1, N + 1) if N % b == 0]


@pytest.mark.parametrize("b,N", _all_pairs(64))
def test_sigma_is_reshape_transpose_flatten(b, N):
    # Sec. 3.1: P reshapes the vector to 2-D (b x N/b), transposes and flattens it.
    s = oracle.perm(b, N)
    want = np.arange(N).reshape(b, N // b).T.ravel()
    assert np.array_equal(s, want)


@pytest.mark.parametrize("b,N", _all_pairs(48))
def test_transpose_rule(b, N):
    # Appendix: P_(b,N)^T = P_(N/b,N); for permutations the transpose is the inverse.
    s = oracle.perm(b, N)
    t = oracle.perm(N // b, N)
    assert np.array_equal(s[t], np.arange(N))
    assert np.array_equal(t[s], np.arange(N))


@pytest.mark.parametrize("b", [1, 2, 3, 4, 8, 16, 32])
def test_square_case_is_involution(b):
    s = oracle.perm(b, b * b)
    assert np.array_equal(s[s], np.arange(b * b))


def test_rejects_non_divisor():
    with pytest.raises(ValueError):
        oracle.perm(3, 10)


def test_worked_values():
    # sigma(i1*b+i0) = i0*N/b + i1, b = 2, N = 6: rows of the 2x3 view interleave.
    assert oracle.perm(2, 6).tolist() == [0, 3, 1, 4, 2, 5]
    assert oracle.perm(3, 6).tolist() == [0, 2, 4, 1, 3, 5]
