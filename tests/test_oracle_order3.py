"""Pins for the oracle's general order-3 Monarch product and its gradients (appendix definition of order-p
Monarch matrices, p = 3): the stepwise form against the dense matrix of the same product (built from dense
permutations and dense block-diagonals by the C oracle), the DFT factors, and the gradients by linearity."""
import numpy as np
import pytest

import oracle
from oracle import order3


def _inputs(b, batch, seed):
    rng = np.random.default_rng(seed)
    N = b ** 3
    f = [rng.standard_normal((b * b, b, b)) / np.sqrt(b) for _ in range(3)]
    return rng.standard_normal((batch, N)), f, rng.standard_normal((batch, N))


@pytest.mark.parametrize("b", [2, 3, 4, 8])
def test_steps_equal_the_dense_product(b):
    x, (B1, B2, B3), _ = _inputs(b, 5, b)
    M = oracle.monarch3_dense(B1, B2, B3)
    assert np.abs(M.imag).max() == 0
    assert np.abs(order3.matmul3(x, B1, B2, B3) - x @ M.real.T).max() < 1e-11


def test_identity_blocks_give_the_sub_index_reversal():
    b = 3
    x, _, _ = _inputs(b, 2, 0)
    eye = np.broadcast_to(np.eye(b), (b * b, b, b))
    y = order3.matmul3(x, eye, eye, eye).reshape(2, b, b, b)
    # factor a moves sub-index a to its mirrored place: the identity blocks leave y[m2,m1,m0] = x[j2=m0, j1=m1, j0=m2]
    assert np.array_equal(y, x.reshape(2, b, b, b).transpose(0, 3, 2, 1))


def test_dft_factors_real_and_imaginary_parts():
    # the blocks that make the order-3 product the DFT: their real parts alone are a real order-3 Monarch matrix
    b = 4
    B1, B2, B3 = oracle.dft3_factors(b)
    x, _, _ = _inputs(b, 3, 1)
    M = oracle.monarch3_dense(B1.real, B2.real, B3.real).real
    assert np.abs(order3.matmul3(x, B1.real, B2.real, B3.real) - x @ M.T).max() < 1e-10


@pytest.mark.parametrize("b", [2, 3, 4])
def test_gradients_by_linearity_in_each_factor(b):
    # S is linear in each factor: dS/dB_k[blk][r][c] = S with B_k replaced by the one-hot E(blk, r, c), through
    # the dense forward matrix
    x, (B1, B2, B3), dy = _inputs(b, 4, 10 + b)
    dx, d1, d2, d3 = order3.matmul3_backward(x, B1, B2, B3, dy)
    S = lambda A1, A2, A3: float(np.sum(dy * (x @ oracle.monarch3_dense(A1, A2, A3).real.T)))
    rng = np.random.default_rng(0)
    for k, got in enumerate((d1, d2, d3)):
        for _ in range(12):
            idx = tuple(rng.integers(0, s) for s in got.shape)
            E = np.zeros_like(B1)
            E[idx] = 1.0
            f = [B1, B2, B3]
            f[k] = E
            assert abs(got[idx] - S(*f)) < 1e-10 * max(1.0, abs(got[idx]))
    M = oracle.monarch3_dense(B1, B2, B3).real
    assert np.abs(dx - dy @ M).max() < 1e-11


def test_gradients_by_central_differences():
    b = 2
    x, (B1, B2, B3), dy = _inputs(b, 3, 5)
    dx, d1, d2, d3 = order3.matmul3_backward(x, B1, B2, B3, dy)
    S = lambda xx, A1, A2, A3: float(np.sum(dy * order3.matmul3(xx, A1, A2, A3)))
    h = 1e-6
    for k, got in enumerate((d1, d2, d3)):
        f = [B1.copy(), B2.copy(), B3.copy()]
        num = np.zeros_like(got)
        for idx in np.ndindex(*got.shape):
            f[k][idx] += h; up = S(x, *f)
            f[k][idx] -= 2 * h; dn = S(x, *f)
            f[k][idx] += h
            num[idx] = (up - dn) / (2 * h)
        assert np.abs(num - got).max() < 1e-7
    e = np.zeros_like(x); e[1, 5] = 1.0
    assert abs((S(x + h * e, B1, B2, B3) - S(x - h * e, B1, B2, B3)) / (2 * h) - dx[1, 5]) < 1e-7


def test_adjoint_identity_and_batch_additivity():
    b = 4
    x, (B1, B2, B3), dy = _inputs(b, 6, 2)
    dx, d1, d2, d3 = order3.matmul3_backward(x, B1, B2, B3, dy)
    assert abs(np.sum(dx * x) - np.sum(dy * order3.matmul3(x, B1, B2, B3))) < 1e-9
    a = order3.matmul3_backward(x[:2], B1, B2, B3, dy[:2])
    c = order3.matmul3_backward(x[2:], B1, B2, B3, dy[2:])
    for k in (1, 2, 3):
        assert np.abs(a[k] + c[k] - (d1, d2, d3)[k - 1]).max() < 1e-10


def test_a_swapped_block_index_is_seen():
    # planted mistake: the blocks of the second factor numbered (j0, m0) instead of (m0, j0)
    b = 3
    x, (B1, B2, B3), _ = _inputs(b, 2, 3)
    wrong = B2.reshape(b, b, b, b).transpose(1, 0, 2, 3).reshape(b * b, b, b)
    M = oracle.monarch3_dense(B1, B2, B3).real
    assert np.abs(order3.matmul3(x, B1, wrong, B3) - x @ M.T).max() > 1e-3
