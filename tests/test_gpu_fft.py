"""GPU parity: monarch_fft / monarch_ifft (Monarch-factored DFT) against the O(N^2) oracle DFT."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL_BF16, TOL_F32, announce, dev, host, rel_l2
from paper_2310_12109_amd import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mm():
    from paper_2310_12109_amd import binding
    return binding


def _cplx(t):
    a = host(t)
    return a[..., 0] + 1j * a[..., 1]


ORDER2 = [(16, 16), (64, 32), (32, 64), (4, 8), (3, 5), (128, 16)]
ORDER3 = [(8, 8, 8), (4, 2, 8), (16, 16, 16), (3, 5, 7)]


@pytest.mark.parametrize("factors", ORDER2 + ORDER3)
@pytest.mark.parametrize("real_input", [True, False])
def test_fft_matches_naive_dft(mm, factors, real_input):
    announce("fft", factors, "real" if real_input else "complex")
    N = int(np.prod(factors))
    rows = 5
    rng = np.random.default_rng(N)
    xr = rng.standard_normal((rows, N)).astype(np.float32)
    xi = rng.standard_normal((rows, N)).astype(np.float32)
    if real_input:
        X = _cplx(mm.monarch_fft(dev(xr), factors, True))
        want = oracle.dft(xr.astype(np.float64))
    else:
        X = _cplx(mm.monarch_fft(dev(np.stack([xr, xi], -1)), factors, False))
        want = oracle.dft(xr.astype(np.float64) + 1j * xi.astype(np.float64))
    assert rel_l2(X, want) <= TOL_F32


@pytest.mark.parametrize("factors", [(16, 16), (64, 32), (8, 8, 8), (3, 5, 7)])
def test_ifft_matches_naive_inverse_and_round_trip(mm, factors):
    announce("ifft", factors)
    N = int(np.prod(factors))
    rng = np.random.default_rng(N + 1)
    Xr = rng.standard_normal((3, N)).astype(np.float32)
    Xi = rng.standard_normal((3, N)).astype(np.float32)
    Xd = dev(np.stack([Xr, Xi], -1))
    x = _cplx(mm.monarch_ifft(Xd, factors, False))
    want = oracle.idft(Xr.astype(np.float64) + 1j * Xi.astype(np.float64))
    assert rel_l2(x, want) <= TOL_F32
    xre = host(mm.monarch_ifft(Xd, factors, True))
    assert rel_l2(xre, want.real) <= TOL_F32
    # inverse(forward(x)) = x
    x0 = rng.standard_normal((3, N)).astype(np.float32)
    back = host(mm.monarch_ifft(mm.monarch_fft(dev(x0), factors, True), factors, True))
    assert rel_l2(back, x0) <= TOL_F32


def test_bf16_input(mm):
    announce("fft bf16 input 64x32")
    x = workloads.round_to_bf16(np.random.default_rng(2).standard_normal((4, 2048)).astype(np.float32))
    X = _cplx(mm.monarch_fft(dev(x, True), (64, 32), True))
    assert rel_l2(X, oracle.dft(x.astype(np.float64))) <= TOL_BF16


MFMA_FACTORS = [(16, 16), (64, 32), (32, 64), (128, 16), (16, 128), (16, 16, 16), (32, 16, 64)]


@pytest.mark.parametrize("factors", MFMA_FACTORS)
@pytest.mark.parametrize("real_input", [True, False])
def test_bf16_fft_matrix_core_passes(mm, factors, real_input):
    # bf16 data with factors of 16..128 take the MFMA passes (bf16 operands, fp32 accumulation)
    announce("fft bf16 mfma", factors, "real" if real_input else "complex")
    N = int(np.prod(factors))
    rows = 3
    rng = np.random.default_rng(N + 11)
    xr = workloads.round_to_bf16(rng.standard_normal((rows, N)).astype(np.float32))
    xi = workloads.round_to_bf16(rng.standard_normal((rows, N)).astype(np.float32))
    if real_input:
        X = _cplx(mm.monarch_fft(dev(xr, True), factors, True))
        want = oracle.dft(xr.astype(np.float64))
    else:
        X = _cplx(mm.monarch_fft(dev(np.stack([xr, xi], -1), True), factors, False))
        want = oracle.dft(xr.astype(np.float64) + 1j * xi.astype(np.float64))
    assert rel_l2(X, want) <= TOL_BF16
    # no row may hide behind the others
    num = np.linalg.norm(X - want, axis=1)
    assert (num / np.linalg.norm(want, axis=1)).max() <= TOL_BF16


@pytest.mark.parametrize("factors", [(16, 16), (64, 32), (128, 128), (16, 32, 16)])
def test_bf16_ifft_matrix_core_passes(mm, factors):
    announce("ifft bf16 mfma", factors)
    N = int(np.prod(factors))
    rng = np.random.default_rng(N + 12)
    Xr = rng.standard_normal((2, N)).astype(np.float32)
    Xi = rng.standard_normal((2, N)).astype(np.float32)
    Xd = dev(np.stack([Xr, Xi], -1))
    spec = Xr.astype(np.float64) + 1j * Xi.astype(np.float64)
    if N <= 4096:
        want = oracle.idft(spec)
    else:   # library routine for the long rows; the paper's forward sign is +, so its inverse is numpy's forward / N
        want = np.fft.fft(spec, axis=-1) / N
    x = _cplx(mm.monarch_ifft(Xd, factors, False, dtype=torch.bfloat16))
    assert rel_l2(x, want) <= TOL_BF16
    xre = host(mm.monarch_ifft(Xd, factors, True, dtype=torch.bfloat16))
    assert rel_l2(xre, want.real) <= TOL_BF16


@pytest.mark.parametrize("factors,rows", [((64, 32), 1300), ((32, 32), 700), ((64, 64), 600), ((128, 64), 300)])
def test_bf16_real_rows_one_kernel_many_rows(mm, factors, rows):
    # real bf16 rows with two LDS-sized factors: one kernel per transform, workgroups walk over several rows;
    # checked against the library FFT (paper's sign: forward = conj of numpy's forward for real input)
    announce("fft/ifft bf16 one kernel", factors, rows)
    N = int(np.prod(factors))
    rng = np.random.default_rng(N + rows)
    x = workloads.round_to_bf16(rng.standard_normal((rows, N)).astype(np.float32))
    X = _cplx(mm.monarch_fft(dev(x, True), factors, True))
    want = np.conj(np.fft.fft(x.astype(np.float64), axis=-1))
    num = np.linalg.norm(X - want, axis=1)
    assert (num / np.linalg.norm(want, axis=1)).max() <= TOL_BF16
    # a few rows against the oracle's own sum as well
    for r in (0, rows // 2, rows - 1):
        assert rel_l2(X[r:r + 1], oracle.dft(x[r:r + 1].astype(np.float64))) <= TOL_BF16
    Xr = rng.standard_normal((rows, N)).astype(np.float32)
    Xi = rng.standard_normal((rows, N)).astype(np.float32)
    back = host(mm.monarch_ifft(dev(np.stack([Xr, Xi], -1)), factors, True, dtype=torch.bfloat16))
    want = (np.fft.fft(Xr.astype(np.float64) + 1j * Xi.astype(np.float64), axis=-1) / N).real
    num = np.linalg.norm(back - want, axis=1)
    assert (num / np.linalg.norm(want, axis=1)).max() <= TOL_BF16


@pytest.mark.parametrize("real_input", [True, False])
def test_bf16_forward_128x128_many_rows(mm, real_input):
    # forward transform of bf16 rows of 16384 = 128 x 128 in one kernel (natural-order spectrum store), more rows
    # than workgroups so that each walks over several: sampled bins of sampled rows against the oracle's own sum,
    # every row against the library FFT (the paper's forward sign is +: the conjugate of numpy's forward on
    # conjugated input)
    announce("fft bf16 128x128 forward", "real" if real_input else "complex")
    N, rows = 16384, 530
    rng = np.random.default_rng(N + rows + int(real_input))
    xr = workloads.round_to_bf16(rng.standard_normal((rows, N)).astype(np.float32))
    if real_input:
        x64 = xr.astype(np.float64)
        X = _cplx(mm.monarch_fft(dev(xr, True), (128, 128), True))
    else:
        xi = workloads.round_to_bf16(rng.standard_normal((rows, N)).astype(np.float32))
        x64 = xr.astype(np.float64) + 1j * xi.astype(np.float64)
        X = _cplx(mm.monarch_fft(dev(np.stack([xr, xi], -1), True), (128, 128), False))
    bins = np.concatenate([[0, 1, 127, 128, N // 2, N - 1], rng.choice(N, size=26, replace=False)]).astype(np.int32)
    for r in (0, 255, 256, rows - 1):
        want = oracle.dft_bins(x64[r:r + 1], bins)
        assert rel_l2(X[r:r + 1, bins], want) <= TOL_BF16
    lib = np.conj(np.fft.fft(np.conj(x64), axis=-1))
    num = np.linalg.norm(X - lib, axis=1)
    assert (num / np.linalg.norm(lib, axis=1)).max() <= TOL_BF16


def test_unit_vector_gives_dft_column(mm):
    announce("fft delta")
    N = 256
    x = np.zeros((1, N), dtype=np.float32); x[0, 3] = 1.0
    X = _cplx(mm.monarch_fft(dev(x), (16, 16), True))[0]
    m = np.arange(N)
    assert np.abs(X - np.exp(2j * np.pi * ((3 * m) % N) / N)).max() < 1e-5


@pytest.mark.parametrize("factors", [(128, 128), (64, 64, 64)])
def test_large_sizes_on_sampled_bins(mm, factors):
    announce("fft large sampled", factors)
    N = int(np.prod(factors))
    rng = np.random.default_rng(7)
    x = rng.standard_normal((2, N)).astype(np.float32)
    X = _cplx(mm.monarch_fft(dev(x), factors, True))
    bins = np.concatenate([[0, 1, N // 2, N - 1], rng.choice(N, size=28, replace=False)]).astype(np.int32)
    want = oracle.dft_bins(x.astype(np.float64), bins)
    assert rel_l2(X[:, bins], want) <= TOL_F32
    # Parseval over the full output: ||F x||^2 = N ||x||^2
    assert np.allclose((np.abs(X) ** 2).sum(-1), N * (x.astype(np.float64) ** 2).sum(-1), rtol=1e-5)


def test_zero_rows(mm):
    announce("fft zero rows")
    X = mm.monarch_fft(torch.empty((0, 256), device="cuda"), (16, 16), True)
    assert X.shape == (0, 256, 2)
