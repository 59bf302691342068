"""GPU parity: monarch_blocky_prepare / monarch_blocky_conv (polynomial-parameterised Monarch matrices, the causal
masks and the Monarch convolution with a general invertible M; appendix) against the numpy oracle."""
import numpy as np
import pytest
import torch

from gpu_util import TOL_BF16, TOL_F32, announce, dev, host, rel_l2
from oracle import blocky
from paper_2310_12109_amd import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mm():
    from paper_2310_12109_amd import binding
    return binding


def _conv(mm, w, b, mask=True, bf16=False):
    state = mm.monarch_blocky_prepare(dev(w["Lt"]), dev(w["Rt"]), dev(w["k"]), mask=mask)
    return mm.monarch_blocky_conv(dev(w["u"], bf16), dev(w["g_in"], bf16), dev(w["g_out"], bf16), state, b)


def _want(w, mask=True):
    return blocky.blocky_monarch_conv(w["Lt"], w["Rt"], w["k"], w["u"], w["g_in"], w["g_out"], mask=mask)[0]


@pytest.mark.parametrize("b,mask", [(4, True), (16, True), (16, False), (32, True)])
def test_prepared_state(mm, b, mask):
    # factors, blockwise inverses (float64 on the GPU, rounded to float32) and the transformed kernels
    announce("blocky prepare b, mask", b, mask)
    H, n = 5, b * (b // 2)
    w = workloads.blocky_inputs(1, H, n, b, seed=b, noise=0.05 if mask else 0.01)
    state = mm.monarch_blocky_prepare(dev(w["Lt"]), dev(w["Rt"]), dev(w["k"]), mask=mask)
    torch.cuda.synchronize()
    R1, L1, R2, L2, Kf = (t.cpu().numpy().astype(np.complex128) for t in mm.blocky_state_views(state, H, b))
    Lt, Rt = blocky.causal_mask(w["Lt"], w["Rt"]) if mask else (w["Lt"], w["Rt"])
    L, R = blocky.blocky_monarch(Lt, Rt)
    wL2, wR2 = blocky.inverse_blocks(L, R)
    for got, want in ((R1, R), (L1, L), (R2, wR2), (L2, wL2)):
        assert rel_l2(got, want) <= 2e-7          # float64 results rounded once to float32
    kp = np.zeros((H, b * b)); kp[:, :n] = w["k"]
    assert rel_l2(Kf, kp @ blocky.dense_from_blocks(L, R).T) <= TOL_F32


@pytest.mark.parametrize("B,H", [(4, 16), (1, 1), (3, 7), (9, 31)])
def test_causal_n128_fp32(mm, B, H):
    announce("blocky conv fp32 b=16 n=128 B,H", B, H)
    w = workloads.blocky_inputs(B, H, 128, 16, seed=B * 10 + H)
    assert rel_l2(host(_conv(mm, w, 16)), _want(w)) <= TOL_F32


@pytest.mark.parametrize("n", [16, 64, 112, 100, 36])
def test_causal_b16_other_lengths(mm, n):
    # multiples of 16 take the matrix-core kernel (dead K steps, partly filled tiles), the others the LDS-tile kernel
    announce("blocky conv fp32 b=16 n", n)
    w = workloads.blocky_inputs(3, 7, n, 16, seed=n)
    assert rel_l2(host(_conv(mm, w, 16)), _want(w)) <= TOL_F32


def test_causal_b16_more_tiles_than_workgroups(mm):
    # 1251 tiles on at most 512 workgroups, the last one ragged
    B, H = 41, 488
    announce("blocky conv fp32 b=16 n=128 B,H", B, H)
    w = workloads.blocky_inputs(B, H, 128, 16, seed=11)
    got, want = host(_conv(mm, w, 16)), _want(w)
    assert rel_l2(got, want) <= TOL_F32
    err = np.linalg.norm(got - want, axis=-1) / np.linalg.norm(want, axis=-1)
    assert err.max() <= 10 * TOL_F32      # no single row is off


@pytest.mark.parametrize("gates", ["in", "out"])
def test_causal_b16_one_gate(mm, gates):
    announce("blocky conv fp32 b=16 gate", gates)
    w = workloads.blocky_inputs(3, 7, 128, 16, seed=5)
    w["g_out" if gates == "in" else "g_in"] = None
    assert rel_l2(host(_conv(mm, w, 16)), _want(w)) <= TOL_F32


@pytest.mark.parametrize("b,n", [(2, 2), (4, 8), (5, 10), (8, 20), (8, 32), (32, 512), (32, 300)])
def test_causal_other_block_sizes_fp32(mm, b, n):
    announce("blocky conv fp32 b, n", b, n)
    w = workloads.blocky_inputs(3, 5, n, b, seed=b + n)
    assert rel_l2(host(_conv(mm, w, b)), _want(w)) <= TOL_F32


@pytest.mark.parametrize("b,n,B,H,gates", [(32, 512, 9, 31, True), (32, 20, 2, 3, True), (32, 302, 2, 3, True), (64, 1000, 3, 7, True),
                                           (64, 2048, 2, 3, False), (32, 512, 40, 13, True)])
def test_blocks_of_32_and_64_in_place_on_the_matrix_cores(mm, b, n, B, H, gates):
    # N = 1024, 4096: the four complex factors in place on two planes of an LDS tile (16 or 4 rows); ragged last tiles,
    # rows of 20 elements (one row tile of the last stage), more tiles than workgroups (520 rows in tiles of 16 on at most
    # 256 workgroups is one tile each: the 40 x 13 case has 33 tiles, the 3 x 7 case at b = 64 six tiles of four rows);
    # n = 302 is not a multiple of 4: the shape-generic kernel
    announce("blocky conv fp32 b, n, B, H", b, n, B, H, gates)
    w = workloads.blocky_inputs(B, H, n, b, seed=b + n + B, noise=0.02 if b == 64 else 0.05, gates=gates)
    assert rel_l2(host(_conv(mm, w, b)), _want(w)) <= TOL_F32


def test_causal_n2048_fp32(mm):
    # b = 64, N = 4096: the largest block size; one row per tile
    announce("blocky conv fp32 b=64 n=2048")
    w = workloads.blocky_inputs(2, 3, 2048, 64, seed=64, noise=0.02)
    assert rel_l2(host(_conv(mm, w, 64)), _want(w)) <= TOL_F32


@pytest.mark.parametrize("b", [8, 16])
def test_unmasked_full_length(mm, b):
    # no mask, n = N: a general (non-causal) invertible M, every input and output index live
    announce("blocky conv fp32 unmasked b", b)
    w = workloads.blocky_inputs(3, 4, b * b, b, seed=b, noise=0.01)
    assert rel_l2(host(_conv(mm, w, b, mask=False)), _want(w, mask=False)) <= TOL_F32


def test_short_kernel_and_no_gates(mm):
    announce("blocky conv fp32 klen < n, no gates")
    w = workloads.blocky_inputs(2, 6, 128, 16, seed=9, klen=37, gates=False)
    assert rel_l2(host(_conv(mm, w, 16)), _want(w)) <= TOL_F32


def test_identity_coefficients_give_the_ordinary_causal_convolution(mm):
    # DFT corollary on the GPU: against the direct convolution sum of the C oracle
    import oracle
    announce("blocky conv fp32 identity coefficients")
    w = workloads.blocky_inputs(2, 4, 128, 16, seed=2, noise=0.0)
    want = oracle.causal_conv(w["u"], w["k"], w["g_in"], w["g_out"])
    assert rel_l2(host(_conv(mm, w, 16)), want) <= TOL_F32


@pytest.mark.parametrize("b,n", [(16, 128), (32, 512)])
def test_bf16(mm, b, n):
    announce("blocky conv bf16 b, n", b, n)
    w = workloads.blocky_inputs(3, 5, n, b, seed=b, bf16=True)
    y = _conv(mm, w, b, bf16=True)
    assert y.dtype == torch.bfloat16
    assert rel_l2(host(y), _want(w)) <= TOL_BF16


@pytest.mark.parametrize("n,B,H", [(128, 7, 93), (48, 3, 7), (256, 2, 5), (16, 3, 5)])
def test_bf16_b16_matrix_core_kernel(mm, n, B, H):
    # bf16 tiles through the matrix-core kernel: many ragged tiles; a tile that fills one and a half load
    # instructions (n = 48); rows longer than 128 (no mask: the lemma allows at most 128 taps); the shortest rows
    announce("blocky conv bf16 b=16 n, B, H", n, B, H)
    mask = n <= 128
    w = workloads.blocky_inputs(B, H, n, 16, seed=n + B, noise=0.05 if mask else 0.01, bf16=True)
    y = _conv(mm, w, 16, mask=mask, bf16=True)
    assert y.dtype == torch.bfloat16
    assert rel_l2(host(y), _want(w, mask=mask)) <= TOL_BF16


def test_output_is_causal_on_the_gpu(mm):
    announce("blocky conv causality")
    w = workloads.blocky_inputs(1, 3, 128, 16, seed=4)
    y0 = host(_conv(mm, w, 16))
    w["u"] = w["u"].copy()
    w["u"][:, :, 77:] += 1.0
    y1 = host(_conv(mm, w, 16))
    scale = np.abs(y0).max()
    assert np.abs(y1[:, :, :77] - y0[:, :, :77]).max() <= 1e-5 * scale   # rounding only: later inputs do enter the arithmetic
    assert np.abs(y1[:, :, 77:] - y0[:, :, 77:]).max() > 1e-2 * scale


def test_empty(mm):
    w = workloads.blocky_inputs(1, 4, 128, 16, seed=0)
    for key in ("u", "g_in", "g_out"):
        w[key] = w[key][:0]
    assert _conv(mm, w, 16).shape == (0, 4, 128)
