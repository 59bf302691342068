"""Pins for the oracle's direct long convolution and the FFT-convolution identity."""
import numpy as np
import pytest

import oracle


@pytest.mark.parametrize("n,klen", [(1, 1), (7, 7), (64, 64), (33, 10), (128, 128)])
def test_direct_sum_against_library_convolve(n, klen):
    rng = np.random.default_rng(n * 100 + klen)
    B, H = 2, 3
    u = rng.standard_normal((B, H, n))
    k = rng.standard_normal((H, klen))
    y = oracle.causal_conv(u, k, nfft=2 * n)
    for b in range(B):
        for h in range(H):
            assert np.abs(y[b, h] - np.convolve(k[h], u[b, h])[:n]).max() < 1e-12


def test_delta_kernels_and_gates():
    rng = np.random.default_rng(0)
    B, H, n = 2, 2, 16
    u = rng.standard_normal((B, H, n))
    gi = rng.standard_normal((B, H, n))
    go = rng.standard_normal((B, H, n))
    k0 = np.zeros((H, n)); k0[:, 0] = 1.0
    k1 = np.zeros((H, n)); k1[:, 1] = 1.0
    assert np.array_equal(oracle.causal_conv(u, k0, gi, go), go * (gi * u))
    y1 = oracle.causal_conv(u, k1)
    assert np.array_equal(y1[..., 1:], u[..., :-1]) and not y1[..., 0].any()


def test_linearity_and_causality():
    rng = np.random.default_rng(1)
    B, H, n = 1, 2, 40
    u1, u2 = rng.standard_normal((2, B, H, n))
    k = rng.standard_normal((H, n))
    y = oracle.causal_conv(2.0 * u1 - 3.0 * u2, k)
    assert np.abs(y - (2.0 * oracle.causal_conv(u1, k) - 3.0 * oracle.causal_conv(u2, k))).max() < 1e-12
    t0 = 17
    u3 = u1.copy(); u3[..., t0:] = rng.standard_normal((B, H, n - t0))
    # Thm 3 (causality): outputs before t0 do not see inputs from t0 on -- exactly.
    assert np.array_equal(oracle.causal_conv(u3, k)[..., :t0], oracle.causal_conv(u1, k)[..., :t0])


@pytest.mark.parametrize("n,nfft", [(4, 8), (16, 32), (16, 48), (64, 128), (30, 64)])
def test_fft_convolution_identity(n, nfft):
    # y = (F^-1((F k') o (F u')))[0:n] with zero padding to nfft >= 2n equals the causal sum.
    rng = np.random.default_rng(n + nfft)
    u = rng.standard_normal(n)
    k = rng.standard_normal(n)
    yf = oracle.fft_conv_row(u, k, nfft)
    yd = oracle.causal_conv(u[None, None], k[None], nfft=nfft)[0, 0]
    assert np.abs(yf[:n].real - yd).max() < 1e-11
    assert np.abs(yf.imag).max() < 1e-11


def test_circular_mode_is_cyclic_convolution():
    # causal=0: kernel of length nfft indexed modulo nfft (negative lags wrapped to the end).
    rng = np.random.default_rng(3)
    n, nfft = 12, 32
    u = rng.standard_normal(n)
    k = rng.standard_normal(nfft)
    y = oracle.causal_conv(u[None, None], k[None], nfft=nfft, causal=False)[0, 0]
    yf = oracle.fft_conv_row(u, k, nfft)
    assert np.abs(yf[:n].real - y).max() < 1e-11
    # two-sided Toeplitz: y[t] = sum_s kk[t-s] u[s], kk[-l] stored at nfft-l
    want = np.array([sum(k[(t - s) % nfft] * u[s] for s in range(n)) for t in range(n)])
    assert np.abs(want - y).max() < 1e-12


def test_monarch_convolution_with_dft_monarch():
    # Alg. 2 with M the order-2 Monarch DFT: f = M^-1 ((M k) o (M u)), zero-padded, equals causal conv.
    rng = np.random.default_rng(4)
    n, N1, N2 = 16, 4, 8
    N = N1 * N2
    M = oracle.monarch_dft_dense(N1, N2)
    u = np.zeros(N); u[:n] = rng.standard_normal(n)
    k = np.zeros(N); k[:n] = rng.standard_normal(n)
    f = np.linalg.solve(M, (M @ k) * (M @ u))
    yd = oracle.causal_conv(u[None, None, :n], k[None, :n], nfft=N)[0, 0]
    assert np.abs(f[:n].real - yd).max() < 1e-11 and np.abs(f.imag).max() < 1e-11


@pytest.mark.parametrize("causal", [True, False])
def test_single_outputs_against_library_convolve_and_a_toeplitz_product(causal):
    # causal_conv_points: y[b, h, t] one output at a time.  Causal: the library's full convolution of the gated
    # row, times the output gate.  Circular (two-sided kernel of length nfft): an explicit Toeplitz matrix
    # T[t, s] = k[(t - s) mod nfft] built with numpy indexing.
    rng = np.random.default_rng(5 + int(causal))
    B, H, n, nfft = 3, 4, 37, 80
    klen = 29 if causal else nfft
    u, gi, go = rng.standard_normal((3, B, H, n))
    k = rng.standard_normal((H, klen))
    rows = rng.integers(0, B * H, size=60)
    ts = rng.integers(0, n, size=60)
    ts[:3] = (0, n - 1, klen % n)
    got = oracle.causal_conv_points(u, k, gi, go, rows, ts, nfft=nfft, causal=causal)
    for i, (row, t) in enumerate(zip(rows, ts)):
        b, h = divmod(int(row), H)
        if causal:
            want = np.convolve(k[h], gi[b, h] * u[b, h])[t] * go[b, h, t]
        else:
            T = k[h][(np.arange(n)[:, None] - np.arange(n)[None, :]) % nfft]
            want = (T @ (gi[b, h] * u[b, h]))[t] * go[b, h, t]
        assert abs(got[i] - want) < 1e-12
    # no gates; a planted off-by-one lag would be seen by the delta kernel
    k1 = np.zeros((H, 5)); k1[:, 1] = 1.0
    pts = oracle.causal_conv_points(u, k1, None, None, [0, 5], [0, 9], nfft=nfft, causal=True)
    assert pts[0] == 0.0 and pts[1] == u[1, 1, 8]     # row 5 = (b 1, h 1)
