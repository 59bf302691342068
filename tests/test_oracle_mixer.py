"""Pins for the oracle's learned-Monarch sequence mixer y = g_out o M2 (K o M1 (g_in o u)) (Sec. 3.2 Eq. 2)."""
import numpy as np
import pytest

import oracle


def _inputs(b, B, H, seed, gates=True):
    rng = np.random.default_rng(seed)
    N = b * b
    u = rng.standard_normal((B, H, N))
    K = rng.standard_normal((H, N))
    gi = rng.standard_normal((B, H, N)) if gates else None
    go = rng.standard_normal((B, H, N)) if gates else None
    f = [rng.standard_normal((b, b, b)) / np.sqrt(b) for _ in range(4)]
    return u, K, gi, go, f


@pytest.mark.parametrize("b", [2, 4, 16])
@pytest.mark.parametrize("gates", [True, False])
def test_against_numpy_with_the_dense_matrices(b, gates):
    u, K, gi, go, (R1, L1, R2, L2) = _inputs(b, 3, 5, b, gates)
    y = oracle.mixer(u, K, gi, go, R1, L1, R2, L2)
    M1, M2 = oracle.monarch_dense(R1, L1), oracle.monarch_dense(R2, L2)
    a = u * gi if gates else u
    t = np.einsum("ij,bhj->bhi", M1, a) * K[None]
    want = np.einsum("ij,bhj->bhi", M2, t)
    if gates:
        want = want * go
    assert np.abs(y - want).max() < 1e-11


def test_identity_blocks_reduce_to_permuted_elementwise_products():
    # L = R = I gives M = P (Sec. 3.1), an involution in the square case: y = P (K o P u) = (P K) o u
    b = 4
    u, K, _, _, _ = _inputs(b, 2, 3, 1, gates=False)
    eye = np.broadcast_to(np.eye(b), (b, b, b)).copy()
    y = oracle.mixer(u, K, None, None, eye, eye, eye, eye)
    s = oracle.perm(b, b * b)
    assert np.array_equal(y, K[:, s][None] * u)


def test_orthogonal_blocks_and_unit_kernel_give_back_the_input():
    # orthogonal blocks make M1 orthogonal; its transpose is the Monarch matrix P R1^T P L1^T P
    # (first factor: transposed blocks of L1, second: those of R1), so with K = 1 the mixer is the identity
    b = 8
    rng = np.random.default_rng(2)
    u = rng.standard_normal((2, 3, b * b))
    q = lambda: np.stack([np.linalg.qr(rng.standard_normal((b, b)))[0] for _ in range(b)])
    R1, L1 = q(), q()
    R2 = np.ascontiguousarray(L1.transpose(0, 2, 1))
    L2 = np.ascontiguousarray(R1.transpose(0, 2, 1))
    y = oracle.mixer(u, np.ones((3, b * b)), None, None, R1, L1, R2, L2)
    assert np.abs(y - u).max() < 1e-12


def test_linear_in_u_and_in_the_kernel_and_channelwise():
    b = 4
    u, K, gi, go, (R1, L1, R2, L2) = _inputs(b, 2, 3, 3)
    f = lambda uu, KK: oracle.mixer(uu, KK, gi, go, R1, L1, R2, L2)
    u2 = np.random.default_rng(4).standard_normal(u.shape)
    assert np.abs(f(2 * u + u2, K) - 2 * f(u, K) - f(u2, K)).max() < 1e-11
    assert np.abs(f(u, 3 * K) - 3 * f(u, K)).max() < 1e-11
    # changing channel 1's kernel changes channel 1 only
    K2 = K.copy()
    K2[1] += 1.0
    d = f(u, K2) - f(u, K)
    assert np.abs(d[:, 0]).max() == 0 and np.abs(d[:, 2]).max() == 0 and np.abs(d[:, 1]).max() > 1e-3
