"""Pins of the oracle of the general order-p Monarch product (Sec. 3.1; appendix definition of the p-variate Monarch
matrix) against what does not depend on its code: the order-2 and order-3 oracles (plain C), the DFT as an order-p
Monarch matrix (naive DFT), the product written digit by digit in Python loops, the reversal as a product of the
paper's permutation family, and exact difference quotients for the gradients."""
import itertools

import numpy as np
import pytest

import oracle
from oracle import orderp


def _factors(b, p, seed=0, complex_=False):
    rng = np.random.default_rng(seed)
    B = rng.standard_normal((p, b ** (p - 1), b, b))
    return B + 1j * rng.standard_normal(B.shape) if complex_ else B


def test_order_two_is_the_order_two_product():
    for b in (2, 3, 4):
        B = _factors(b, 2, seed=b)
        np.testing.assert_allclose(orderp.orderp_dense(B), oracle.monarch_dense(B[0], B[1]), rtol=1e-12, atol=1e-12)


def test_order_three_is_the_order_three_product():
    for b in (2, 3, 4):
        B = _factors(b, 3, seed=10 + b, complex_=True)
        np.testing.assert_allclose(orderp.orderp_dense(B), oracle.monarch3_dense(B[0], B[1], B[2]), rtol=1e-12, atol=1e-12)


def _dft_factors(b, p):
    """omega_N^(m j) = prod over digit pairs (a, c) with a + c < p of omega_N^(m_a j_c b^(a+c)); factor s takes the
    terms of the input digit it consumes, j_(p-s), with every output digit produced up to then (m_0 .. m_(s-1))."""
    N = b ** p
    B = np.zeros((p, b ** (p - 1), b, b), dtype=np.complex128)
    for s in range(1, p + 1):
        for K, key in enumerate(itertools.product(range(b), repeat=p - 1)):      # most significant digit first
            m_done = key[:s - 1]                                                   # m_0 .. m_(s-2)
            for r in range(b):
                ms = list(m_done) + [r]                                            # m_0 .. m_(s-1)
                for c in range(b):
                    e = sum(ms[a] * c * b ** (a + p - s) for a in range(s))
                    B[s - 1, K, r, c] = np.exp(-2j * np.pi * (e % N) / N)
    return B


@pytest.mark.parametrize("b,p", [(2, 2), (2, 4), (3, 4), (2, 6), (4, 4), (2, 5)])
def test_dft_is_an_order_p_monarch_matrix(b, p):
    N = b ** p
    F = np.fft.fft(np.eye(N), axis=0)
    np.testing.assert_allclose(orderp.orderp_dense(_dft_factors(b, p)), F, rtol=1e-10, atol=1e-10)


def _by_digits(x, B):
    """The product one factor at a time in Python loops over digit tuples: the vector between the factors is indexed
    by (produced output digits .., unconsumed input digits .., newest output digit)."""
    p, _, b, _ = B.shape
    digits = lambda n: list(itertools.product(range(b), repeat=n))
    t = {tuple(reversed(j)): x[sum(d * b ** (p - 1 - a) for a, d in enumerate(j))] for j in digits(p)}   # key (j_0 .. j_(p-1))
    for s in range(1, p + 1):
        out = {}
        for m_done in digits(s - 1):                      # m_0 .. m_(s-2)
            for j_left in digits(p - s):                  # j_0 .. j_(p-s-1)
                key = m_done + j_left
                K = sum(d * b ** (p - 2 - a) for a, d in enumerate(key))
                for r in range(b):
                    acc = 0.0
                    for c in range(b):
                        src = m_done[:-1] + j_left + (c,) + m_done[-1:] if s > 1 else j_left + (c,)
                        acc += B[s - 1, K, r, c] * t[src]
                    out[key + (r,)] = acc
        t = out
    y = np.zeros(b ** p, dtype=np.result_type(x, B))
    for m in digits(p):                                   # key (m_0 .. m_(p-1)) -> index sum m_a b^a
        y[sum(d * b ** a for a, d in enumerate(m))] = t[m]
    return y


@pytest.mark.parametrize("b,p", [(2, 4), (3, 3), (2, 5), (3, 4)])
def test_product_digit_by_digit(b, p):
    B = _factors(b, p, seed=p)
    x = np.random.default_rng(1).standard_normal(b ** p)
    np.testing.assert_allclose(orderp.matmulp(x[None], B)[0], _by_digits(x, B), rtol=1e-11, atol=1e-11)


def test_reversal_is_the_product_of_the_permutation_family():
    # P^R = P_(b, b^2, N) P_(b^2, b^3, N) ... P_(b^(p-1), b^p, N) with (P x)[i] = x[sigma[i]]
    for b, p in ((2, 4), (3, 3), (2, 5)):
        N = b ** p
        x = np.arange(N)
        for a in range(p - 1, 0, -1):                     # the rightmost permutation acts first
            x = x[orderp.sigma(b ** a, b ** (a + 1), N)]
        np.testing.assert_array_equal(x, orderp.reversal(b, p))
        assert np.array_equal(orderp.reversal(b, p)[orderp.reversal(b, p)], np.arange(N))


@pytest.mark.parametrize("b,p", [(2, 4), (3, 3), (4, 2)])
def test_gradients_by_exact_difference_quotients(b, p):
    rng = np.random.default_rng(7)
    B = _factors(b, p, seed=3)
    N = b ** p
    x, dy = rng.standard_normal((5, N)), rng.standard_normal((5, N))
    dx, dB = orderp.matmulp_backward(x, B, dy)
    S = lambda xx, BB: float(np.sum(dy * orderp.matmulp(xx, BB)))
    # S is linear in x and in every single factor: the difference quotient with a unit step is the derivative
    for _ in range(12):
        v, j = rng.integers(5), rng.integers(N)
        x2 = x.copy(); x2[v, j] += 1.0
        assert abs(S(x2, B) - S(x, B) - dx[v, j]) < 1e-9
        s, k, r, c = rng.integers(p), rng.integers(b ** (p - 1)), rng.integers(b), rng.integers(b)
        B2 = B.copy(); B2[s, k, r, c] += 1.0
        assert abs(S(x, B2) - S(x, B) - dB[s, k, r, c]) < 1e-9
    # the adjoint identity <dy, M x> = <M^T dy, x>
    assert abs(np.sum(dy * orderp.matmulp(x, B)) - np.sum(dx * x)) < 1e-9


def test_gradients_of_order_three_are_those_of_the_order_three_oracle():
    from oracle import order3
    b = 3
    B = _factors(b, 3, seed=4)
    rng = np.random.default_rng(2)
    x, dy = rng.standard_normal((4, 27)), rng.standard_normal((4, 27))
    dx, dB = orderp.matmulp_backward(x, B, dy)
    want = order3.matmul3_backward(x, B[0], B[1], B[2], dy)
    np.testing.assert_allclose(dx, want[0], rtol=1e-11, atol=1e-11)
    for s in range(3):
        np.testing.assert_allclose(dB[s], want[1 + s], rtol=1e-11, atol=1e-11)
