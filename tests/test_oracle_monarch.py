"""Pins for the oracle's dense order-2 Monarch matrix M = P L P R P (Sec. 3.1)."""
import numpy as np
import pytest
import torch

import oracle


def _pmat(b, N):
    s = np.arange(N).reshape(b, N // b).T.ravel()
    P = np.zeros((N, N))
    P[np.arange(N), s] = 1.0
    return P


def _blockdiag(W):
    nb, o, i = W.shape
    D = np.zeros((nb * o, nb * i), dtype=W.dtype)
    for k in range(nb):
        D[k * o:(k + 1) * o, k * i:(k + 1) * i] = W[k]
    return D


@pytest.mark.parametrize("b", [2, 3, 4, 8, 16])
def test_closed_form_entries_square(b):
    # Appendix Eq. for M' = Lbar R with Lbar = P^T L P, and M = M' P:
    # M'[(i1,i0),(j1,j0)] = Lbar_{i1,j1}[i0,i0] * R_{j1,j1}[i0,j0].
    rng = np.random.default_rng(b)
    N = b * b
    R = rng.standard_normal((b, b, b))
    L = rng.standard_normal((b, b, b))
    M = oracle.monarch_dense(R, L)
    P = _pmat(b, N)
    Mprime = M @ P.T                     # M = M' P  =>  M' = M P^T
    Lbar = P.T @ _blockdiag(L) @ P       # L = P Lbar P^T
    Rd = _blockdiag(R)
    for i1 in range(b):
        for i0 in range(b):
            for j1 in range(b):
                for j0 in range(b):
                    want = Lbar[i1 * b + i0, j1 * b + i0] * Rd[j1 * b + i0, j1 * b + j0]
                    assert abs(Mprime[i1 * b + i0, j1 * b + j0] - want) < 1e-13


@pytest.mark.parametrize("b", [2, 4, 16])
def test_entry_formula_in_block_terms(b):
    # The same closed form spelt with block/row/col of the stored factors:
    # M[i1*b+i0, j1*b+j0] = L_{i0}[i1,j0] * R_{j0}[i0,j1].
    rng = np.random.default_rng(100 + b)
    R = rng.standard_normal((b, b, b))
    L = rng.standard_normal((b, b, b))
    M = oracle.monarch_dense(R, L).reshape(b, b, b, b)   # [i1,i0,j1,j0]
    want = np.einsum("bad,dbc->abcd", L, R)              # L[i0][i1,j0] * R[j0][i0,j1] -> [i1,i0,j1,j0]
    assert np.abs(M - want).max() < 1e-13


@pytest.mark.parametrize("b", [2, 4, 8])
def test_stepwise_application_with_explicit_loops(b):
    # The product applied to a vector one step at a time, every step an explicit loop over (block, row):
    # gather by P, block-diagonal R, gather by P, block-diagonal L, gather by P (Sec. 3.1; the basic layer of the
    # appendix applies the same five steps, with its first-applied factor in the role of R here).
    rng = np.random.default_rng(7 + b)
    N = b * b
    R = rng.standard_normal((b, b, b))
    L = rng.standard_normal((b, b, b))
    sigma = [(i % b) * b + i // b for i in range(N)]         # (P x)[i] = x[sigma(i)]

    def gather(v):
        return [v[sigma[i]] for i in range(N)]

    def blocks(v, W):
        out = [0.0] * N
        for k in range(b):
            for r in range(b):
                out[k * b + r] = sum(W[k, r, c] * v[k * b + c] for c in range(b))
        return out

    M = oracle.monarch_dense(R, L)
    for col in range(N):
        e = [1.0 if j == col else 0.0 for j in range(N)]
        y = gather(blocks(gather(blocks(gather(e), R)), L))
        assert np.abs(M[:, col] - np.array(y)).max() < 1e-13


@pytest.mark.parametrize("b", [2, 3, 5, 16])
def test_identity_blocks_give_permutation(b):
    I = np.tile(np.eye(b), (b, 1, 1))
    M = oracle.monarch_dense(I, I)
    # P P P = P for the involution P_(b,b^2)
    assert np.array_equal(M, _pmat(b, b * b))


def test_identity_blocks_rectangular():
    nbR, r, nbL, l = 3, 4, 6, 2       # d = 12 everywhere
    M = oracle.monarch_dense(np.tile(np.eye(r), (nbR, 1, 1)), np.tile(np.eye(l), (nbL, 1, 1)))
    want = _pmat(nbL, 12) @ _pmat(nbR, 12) @ _pmat(r, 12)
    assert np.array_equal(M, want)


@pytest.mark.parametrize("b", [2, 3, 4])
def test_kronecker_special_case(b):
    # With all blocks of R equal to A and all blocks of L equal to B,
    # P (I x B) P (I x A) P = (B x I)(I x A) P = (B x A) P.
    rng = np.random.default_rng(b)
    A = rng.standard_normal((b, b))
    B = rng.standard_normal((b, b))
    M = oracle.monarch_dense(np.tile(A, (b, 1, 1)), np.tile(B, (b, 1, 1)))
    assert np.abs(M - np.kron(B, A) @ _pmat(b, b * b)).max() < 1e-13


@pytest.mark.parametrize("shape", [(4, 3, 2, 2, 5, 6), (2, 6, 3, 4, 5, 3), (4, 192 // 16, 12, 4, 7, 12)])
def test_rectangular_stepwise(shape):
    # Vector-at-a-time application of the five steps must equal the dense matrix.
    nbR, r_out, r_in, nbL, l_out, l_in = shape
    assert nbR * r_out == nbL * l_in
    rng = np.random.default_rng(sum(shape))
    R = rng.standard_normal((nbR, r_out, r_in))
    L = rng.standard_normal((nbL, l_out, l_in))
    d_in, d_mid, d_out = nbR * r_in, nbR * r_out, nbL * l_out
    x = rng.standard_normal(d_in)
    t0 = x.reshape(r_in, nbR).T                        # P_(r_in,d_in): [k, c]
    t1 = np.einsum("krc,kc->kr", R, t0)                # block k
    t2 = t1.reshape(nbR, r_out).T.reshape(nbL, l_in)   # P_(nbR,d_mid), regrouped for L
    t3 = np.einsum("kra,ka->kr", L, t2)
    y = t3.reshape(nbL, l_out).T.ravel()               # P_(nbL,d_out)
    M = oracle.monarch_dense(R, L)
    assert M.shape == (d_out, d_in) and d_mid == nbL * l_in
    assert np.abs(M @ x - y).max() < 1e-12
    assert np.abs(oracle.matmul(x[None], R, L)[0] - y).max() < 1e-12


def test_matmul_is_dense_matrix_times_vector():
    rng = np.random.default_rng(0)
    R = rng.standard_normal((16, 16, 16)) / 4
    L = rng.standard_normal((16, 16, 16)) / 4
    x = rng.standard_normal((5, 256))
    assert np.abs(oracle.matmul(x, R, L) - x @ oracle.monarch_dense(R, L).T).max() < 1e-12


def test_inconsistent_shapes_rejected():
    with pytest.raises(ValueError):
        oracle.monarch_dense(np.zeros((2, 3, 3)), np.zeros((2, 2, 2)))
