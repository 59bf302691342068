"""Pins for the oracle's gradients of the order-2 Monarch product (Sec. 3.1, M = P L P R P): the chain-rule
code in oracle_matmul_backward is checked against what does not depend on it."""
import numpy as np
import pytest

import oracle

SHAPES = [  # nbR, r_out, r_in, nbL, l_out, l_in
    (4, 4, 4, 4, 4, 4),        # the paper's square case, b = 4
    (2, 6, 3, 4, 5, 3),        # rectangular, d_in 6 -> d_mid 12 -> d_out 20
    (3, 2, 5, 2, 7, 3),        # blocks of different counts
    (16, 16, 16, 16, 16, 16),  # config 1
]


def _rand(shape, seed):
    nbR, r_out, r_in, nbL, l_out, l_in = shape
    rng = np.random.default_rng(seed)
    batch = 5
    x = rng.standard_normal((batch, nbR * r_in))
    R = rng.standard_normal((nbR, r_out, r_in))
    L = rng.standard_normal((nbL, l_out, l_in))
    dy = rng.standard_normal((batch, nbL * l_out))
    return x, R, L, dy


def _S(x, R, L, dy):
    return float((oracle.matmul(x, R, L) * dy).sum())


@pytest.mark.parametrize("shape", SHAPES)
def test_dx_is_the_transposed_dense_matrix(shape):
    x, R, L, dy = _rand(shape, 1)
    dx, _, _ = oracle.matmul_backward(x, R, L, dy)
    M = oracle.monarch_dense(R, L)
    assert np.abs(dx - dy @ M).max() < 1e-12


@pytest.mark.parametrize("shape", SHAPES)
def test_adjoint_identity(shape):
    # <dy, M x> = <M^T dy, x>
    x, R, L, dy = _rand(shape, 2)
    dx, _, _ = oracle.matmul_backward(x, R, L, dy)
    assert abs(_S(x, R, L, dy) - float((dx * x).sum())) < 1e-10 * max(1.0, abs(_S(x, R, L, dy)))


@pytest.mark.parametrize("shape", SHAPES[:3])
def test_parameter_gradients_are_the_map_at_one_hot_factors(shape):
    # S is linear in R for fixed L (and in L for fixed R): dS/dR_k[r,c] = S evaluated with R replaced by the
    # one-hot factor E_(k,r,c), and likewise for L.  Uses only the dense forward oracle.
    x, R, L, dy = _rand(shape, 3)
    _, dR, dL = oracle.matmul_backward(x, R, L, dy)
    for idx in np.ndindex(*R.shape):
        E = np.zeros_like(R)
        E[idx] = 1.0
        assert abs(dR[idx] - _S(x, E, L, dy)) < 1e-11
    for idx in np.ndindex(*L.shape):
        E = np.zeros_like(L)
        E[idx] = 1.0
        assert abs(dL[idx] - _S(x, R, E, dy)) < 1e-11


def test_config1_gradients_on_sampled_entries():
    # the same definition at b = 16 on a sample of entries (all of them would take minutes)
    x, R, L, dy = _rand(SHAPES[3], 4)
    _, dR, dL = oracle.matmul_backward(x, R, L, dy)
    rng = np.random.default_rng(5)
    for _ in range(24):
        idx = tuple(int(rng.integers(0, 16)) for _ in range(3))
        E = np.zeros_like(R)
        E[idx] = 1.0
        assert abs(dR[idx] - _S(x, E, L, dy)) < 1e-10
        assert abs(dL[idx] - _S(x, R, E, dy)) < 1e-10


@pytest.mark.parametrize("shape", SHAPES[:3])
def test_central_differences(shape):
    # S is bilinear in (R, L): a central difference in one entry is exact up to rounding
    x, R, L, dy = _rand(shape, 6)
    dx, dR, dL = oracle.matmul_backward(x, R, L, dy)
    h = 0.5
    rng = np.random.default_rng(7)
    for _ in range(10):
        i = tuple(int(rng.integers(0, n)) for n in R.shape)
        Rp, Rm = R.copy(), R.copy()
        Rp[i] += h
        Rm[i] -= h
        assert abs((_S(x, Rp, L, dy) - _S(x, Rm, L, dy)) / (2 * h) - dR[i]) < 1e-10
        j = tuple(int(rng.integers(0, n)) for n in L.shape)
        Lp, Lm = L.copy(), L.copy()
        Lp[j] += h
        Lm[j] -= h
        assert abs((_S(x, R, Lp, dy) - _S(x, R, Lm, dy)) / (2 * h) - dL[j]) < 1e-10
        q = tuple(int(rng.integers(0, n)) for n in x.shape)
        xp, xm = x.copy(), x.copy()
        xp[q] += h
        xm[q] -= h
        assert abs((_S(xp, R, L, dy) - _S(xm, R, L, dy)) / (2 * h) - dx[q]) < 1e-10


@pytest.mark.parametrize("b", [2, 4, 16])
def test_square_case_dx_is_a_monarch_product_of_the_transposed_blocks(b):
    # square case: P1 = P2 = P3 = P with P^T = P, so M^T = P R^T P L^T P: the order-2 product whose first factor
    # holds the transposed blocks of L and whose second holds those of R
    x, R, L, dy = _rand((b, b, b, b, b, b), 8)
    dx, _, _ = oracle.matmul_backward(x, R, L, dy)
    want = oracle.matmul(dy, np.ascontiguousarray(L.transpose(0, 2, 1)), np.ascontiguousarray(R.transpose(0, 2, 1)))
    assert np.abs(dx - want).max() < 1e-12


def test_identity_blocks_and_batch_additivity():
    b = 4
    x, R, L, dy = _rand((b, b, b, b, b, b), 9)
    eye = np.broadcast_to(np.eye(b), (b, b, b)).copy()
    dx, _, _ = oracle.matmul_backward(x, eye, eye, dy)
    s = oracle.perm(b, b * b)                      # M = P P P = P: y[i] = x[s[i]], so dx[s[i]] = dy[i]
    want = np.zeros_like(dx)
    want[:, s] = dy
    assert np.array_equal(dx, want)
    _, dR, dL = oracle.matmul_backward(x, R, L, dy)
    _, dRa, dLa = oracle.matmul_backward(x[:2], R, L, dy[:2])
    _, dRb, dLb = oracle.matmul_backward(x[2:], R, L, dy[2:])
    assert np.abs(dR - dRa - dRb).max() < 1e-12 and np.abs(dL - dLa - dLb).max() < 1e-12


def test_a_wrong_transpose_would_be_caught():
    # plant the classic mistake (forgetting to transpose a block) in a copy of the result: the pins above see it
    x, R, L, dy = _rand((4, 4, 4, 4, 4, 4), 10)
    _, dR, _ = oracle.matmul_backward(x, R, L, dy)
    wrong = dR.transpose(0, 2, 1)
    E = np.zeros_like(R)
    E[1, 2, 3] = 1.0
    assert abs(dR[1, 2, 3] - _S(x, E, L, dy)) < 1e-11
    assert abs(wrong[1, 2, 3] - _S(x, E, L, dy)) > 1e-6
