"""Pins for the oracle's Monarch MLP y = W2 act(W1 x + b1) + b2 (Sec. 3.2, Eq. 3)."""
import numpy as np
import pytest
from scipy.special import erf

import oracle


def _gelu(z):
    return 0.5 * z * (1.0 + erf(z / np.sqrt(2.0)))


def test_gelu_values_are_z_times_normal_cdf():
    # act(z) = z * Phi(z); Phi(1) = 0.8413447460685429, Phi(-1) = 0.15865525393145707, Phi(0) = 0.5
    x = np.array([[1.0, -1.0, 0.0, 2.0]])
    W = np.eye(4)[None]                      # one 4x4 identity block
    y = oracle.mlp(x, W, None, None, W, None, None, nb=1, order=1, act=2)
    want = np.array([0.8413447460685429, -0.15865525393145707, 0.0, 2 * 0.9772498680518208])
    assert np.abs(y[0] - want).max() < 1e-15


@pytest.mark.parametrize("act", [0, 1, 2])
def test_single_block_is_a_dense_mlp(act):
    rng = np.random.default_rng(act)
    d, dh, T = 6, 10, 5
    x = rng.standard_normal((T, d))
    W1 = rng.standard_normal((1, dh, d)); b1 = rng.standard_normal(dh)
    W2 = rng.standard_normal((1, d, dh)); b2 = rng.standard_normal(d)
    z = x @ W1[0].T + b1
    hcur = {0: z, 1: np.maximum(z, 0), 2: _gelu(z)}[act]
    want = hcur @ W2[0].T + b2
    y = oracle.mlp(x, W1, None, b1, W2, None, b2, nb=1, order=1, act=act)
    assert np.abs(y - want).max() < 1e-12


def test_zero_weights_give_bias():
    d, dh, nb = 8, 16, 4
    x = np.random.default_rng(0).standard_normal((3, d))
    b2 = np.arange(d, dtype=float)
    y = oracle.mlp(x, np.zeros((nb, dh // nb, d // nb)), None, None,
                   np.zeros((nb, d // nb, dh // nb)), None, b2, nb=nb, order=1, act=2)
    assert np.array_equal(y, np.tile(b2, (3, 1)))


def test_order1_blocks_are_independent():
    rng = np.random.default_rng(1)
    d, dh, nb = 12, 24, 3
    W1 = rng.standard_normal((nb, dh // nb, d // nb)); W2 = rng.standard_normal((nb, d // nb, dh // nb))
    x = rng.standard_normal((2, d))
    y0 = oracle.mlp(x, W1, None, None, W2, None, None, nb=nb, order=1, act=2)
    x2 = x.copy(); x2[:, 4:8] += 1.0          # block 1's inputs only
    y1 = oracle.mlp(x2, W1, None, None, W2, None, None, nb=nb, order=1, act=2)
    assert np.array_equal(y0[:, :4], y1[:, :4]) and np.array_equal(y0[:, 8:], y1[:, 8:])
    assert np.abs(y0[:, 4:8] - y1[:, 4:8]).min() > 0
    # and each block is its own small dense MLP
    for k in range(nb):
        want = _gelu(x[:, 4 * k:4 * k + 4] @ W1[k].T) @ W2[k].T
        assert np.abs(y0[:, 4 * k:4 * k + 4] - want).max() < 1e-12


def test_order2_layers_are_the_dense_monarch_matrices():
    rng = np.random.default_rng(2)
    d, dh, nb = 8, 32, 4
    W1R = rng.standard_normal((nb, d // nb, d // nb)); W1L = rng.standard_normal((nb, dh // nb, d // nb))
    W2R = rng.standard_normal((nb, d // nb, dh // nb)); W2L = rng.standard_normal((nb, d // nb, d // nb))
    b1 = rng.standard_normal(dh); b2 = rng.standard_normal(d)
    x = rng.standard_normal((4, d))
    W1 = oracle.monarch_dense(W1R, W1L)
    W2 = oracle.monarch_dense(W2R, W2L)
    assert W1.shape == (dh, d) and W2.shape == (d, dh)
    want = _gelu(x @ W1.T + b1) @ W2.T + b2
    y = oracle.mlp(x, W1R, W1L, b1, W2R, W2L, b2, nb=nb, order=2, act=2)
    assert np.abs(y - want).max() < 1e-12
