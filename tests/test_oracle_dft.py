"""Pins for the oracle's DFT, its Monarch factorisations (order 2 and 3) and the inverse."""
import numpy as np
import pytest

import oracle


def _F(N):
    j = np.arange(N)
    return np.exp(2j * np.pi * ((j[:, None] * j[None, :]) % N) / N)   # paper sign: omega = e^{+2 pi i/N}


@pytest.mark.parametrize("N", [1, 2, 3, 8, 30, 256, 1000])
def test_dft_against_library_fft(N):
    # numpy's inverse transform uses e^{+2 pi i m j / N} / N, i.e. the paper's sign.
    rng = np.random.default_rng(N)
    x = rng.standard_normal((3, N)) + 1j * rng.standard_normal((3, N))
    X = oracle.dft(x)
    assert np.abs(X - N * np.fft.ifft(x, axis=-1)).max() < 1e-9 * max(1, N)
    assert np.abs(oracle.idft(X) - x).max() < 1e-11


def test_dft_of_unit_vectors_gives_columns():
    N = 12
    X = oracle.dft(np.eye(N))
    assert np.abs(X.T - _F(N)).max() < 1e-13     # row r of X is F e_r = column r of F


def test_sign_convention_on_a_shifted_delta():
    # F e_1 = (omega^0, omega^1, ...): the imaginary part of entry 1 is +sin(2 pi/N).
    N = 8
    X = oracle.dft(np.eye(N)[1][None])[0]
    assert X[1].imag == pytest.approx(np.sin(2 * np.pi / N), abs=1e-15)
    assert X[1].real == pytest.approx(np.cos(2 * np.pi / N), abs=1e-15)


@pytest.mark.parametrize("N", [16, 100, 2048])
def test_parseval_and_hermitian_symmetry(N):
    rng = np.random.default_rng(N)
    x = rng.standard_normal((2, N))
    X = oracle.dft(x)
    assert np.allclose((np.abs(X) ** 2).sum(-1), N * (x ** 2).sum(-1), rtol=1e-12)
    assert np.abs(X[:, 1:] - np.conj(X[:, 1:][:, ::-1])).max() < 1e-9   # real input


def test_inverse_is_conjugate_over_N():
    N = 24
    rng = np.random.default_rng(1)
    X = rng.standard_normal((1, N)) + 1j * rng.standard_normal((1, N))
    assert np.abs(oracle.idft(X) - (np.conj(_F(N)) @ X[0]) / N).max() < 1e-13


@pytest.mark.parametrize("N1,N2", [(2, 2), (4, 4), (8, 8), (16, 16), (2, 4), (4, 2), (4, 8), (8, 4),
                                   (3, 5), (32, 8), (64, 32), (32, 64)])
def test_order2_monarch_dft_equals_dense_dft(N1, N2):
    # DFT corollary of the appendix: a particular (L, R) makes P L P R P = F_N.
    M = oracle.monarch_dft_dense(N1, N2)
    assert np.abs(M - _F(N1 * N2)).max() < 1e-10


def test_dft_factor_values():
    R, L = oracle.dft_factors(4, 8)
    assert R.shape == (8, 4, 4) and L.shape == (4, 8, 8)
    for a in range(8):
        assert np.abs(R[a] - _F(4)).max() < 1e-15
    i, k, a = 3, 5, 6
    want = np.exp(2j * np.pi * k * a / 8) * np.exp(2j * np.pi * i * a / 32)
    assert abs(L[i, k, a] - want) < 1e-14


@pytest.mark.parametrize("b", [2, 4, 8])
def test_plain_kronecker_dft_blocks_are_not_the_dft(b):
    # L = R = I (x) F_b omits the twiddle factors: that product is a 2-D DFT, not F_N.
    Fb = np.tile(_F(b), (b, 1, 1))
    M = oracle.monarch_dense(Fb, Fb)
    assert np.abs(M - _F(b * b)).max() > 0.5
    P = oracle.perm(b, b * b)
    assert np.abs(M - np.kron(_F(b), _F(b))[:, P]).max() < 1e-12


@pytest.mark.parametrize("b", [2, 3, 4, 8])
def test_order3_monarch_dft_equals_dense_dft(b):
    M = oracle.monarch3_dft_dense(b)
    assert np.abs(M - _F(b ** 3)).max() < 1e-10


@pytest.mark.parametrize("b", [2, 3, 4])
def test_order3_identity_blocks_give_subindex_reversal(b):
    # P^R P_(b,b^2,N) P_(b^2,b^3,N) P^R = (P^R)^3 = P^R: digits (i2,i1,i0) -> (i0,i1,i2).
    I = np.tile(np.eye(b), (b * b, 1, 1))
    M = oracle.monarch3_dense(I, I, I)
    N = b ** 3
    i = np.arange(N)
    rev = (i % b) * b * b + ((i // b) % b) * b + i // (b * b)
    want = np.zeros((N, N))
    want[i, rev] = 1.0
    assert np.array_equal(M.real, want) and not M.imag.any()


def test_order3_random_blocks_against_digitwise_application():
    # Three rounds of "contract the least significant digit" with the stated permutations.
    b = 3
    N = b ** 3
    rng = np.random.default_rng(5)
    B = [rng.standard_normal((b * b, b, b)) + 1j * rng.standard_normal((b * b, b, b)) for _ in range(3)]
    x = rng.standard_normal(N) + 1j * rng.standard_normal(N)
    v = x.reshape(b, b, b).transpose(2, 1, 0)                 # P^R: [j0,j1,j2]
    v = np.einsum("pqrc,pqc->pqr", B[0].reshape(b, b, b, b), v)   # -> [j0,j1,m0]
    v = v.transpose(2, 0, 1)                                  # P_(b^2,b^3): [m0,j0,j1]
    v = np.einsum("pqrc,pqc->pqr", B[1].reshape(b, b, b, b), v)   # -> [m0,j0,m1]
    v = v.transpose(0, 2, 1)                                  # P_(b,b^2,N): [m0,m1,j0]
    v = np.einsum("pqrc,pqc->pqr", B[2].reshape(b, b, b, b), v)   # -> [m0,m1,m2]
    y = v.transpose(2, 1, 0).ravel()                          # P^R: [m2,m1,m0]
    M = oracle.monarch3_dense(*B)
    assert np.abs(M @ x - y).max() < 1e-12


def test_selected_bins_match_full_transform_and_library():
    rng = np.random.default_rng(9)
    x = rng.standard_normal((2, 4096)) + 1j * rng.standard_normal((2, 4096))
    bins = [0, 1, 17, 2048, 4095]
    Xb = oracle.dft_bins(x, bins)
    assert np.abs(Xb - (4096 * np.fft.ifft(x, axis=-1))[:, bins]).max() < 1e-8
    y = rng.standard_normal((1, 64)) + 0j
    assert np.array_equal(oracle.dft_bins(y, np.arange(64)), oracle.dft(y))
