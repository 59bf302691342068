"""GPU parity: monarch_matmul (order-2 Monarch product, Sec. 3.1) against the dense oracle."""
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


@pytest.mark.parametrize("batch", [64, 67, 1, 1000])
def test_config1_square_fp32(mm, batch):
    announce("matmul c1 fp32 batch", batch)
    w = workloads.monarch_matmul_inputs(batch=batch, b=16, seed=0)
    y = host(mm.monarch_matmul(dev(w["x"]), dev(w["R"]), dev(w["L"])))
    want = oracle.matmul(w["x"], w["R"], w["L"])
    assert rel_l2(y, want) <= TOL_F32


def test_empty_batch(mm):
    announce("matmul empty batch")
    w = workloads.monarch_matmul_inputs(batch=1, b=16, seed=0)
    x = torch.empty((0, 256), device="cuda")
    y = mm.monarch_matmul(x, dev(w["R"]), dev(w["L"]))
    assert y.shape == (0, 256)


@pytest.mark.parametrize("b", [2, 8, 32, 64])
def test_square_other_block_sizes(mm, b):
    announce("matmul square b", b)
    w = workloads.monarch_matmul_inputs(batch=19, b=b, seed=b)
    y = host(mm.monarch_matmul(dev(w["x"]), dev(w["R"]), dev(w["L"])))
    assert rel_l2(y, oracle.matmul(w["x"], w["R"], w["L"])) <= TOL_F32


@pytest.mark.parametrize("b,batch,bf16", [(32, 1, False), (32, 16, False), (32, 1100, False), (64, 8, False), (64, 523, False),
                                          (32, 77, True), (64, 77, True)])
def test_square_blocks_of_32_and_64_in_place_on_the_matrix_cores(mm, b, batch, bf16):
    # tiles of 16 (b = 32) or 8 (b = 64) rows: one row, one tile, ragged tails, more tiles than workgroups
    announce("matmul in place b, batch, bf16", b, batch, bf16)
    w = workloads.monarch_matmul_inputs(batch=batch, b=b, seed=b + batch, bf16=bf16)
    y = host(mm.monarch_matmul(dev(w["x"], bf16), dev(w["R"], bf16), dev(w["L"], bf16)))
    assert rel_l2(y, oracle.matmul(w["x"], w["R"], w["L"])) <= (TOL_BF16 if bf16 else TOL_F32)


@pytest.mark.parametrize("shape", [(4, 3, 2, 2, 5, 6), (4, 192, 192, 4, 768, 192), (4, 192, 768, 4, 192, 192),
                                   (16, 64, 64, 16, 256, 64), (3, 7, 5, 7, 2, 3)])
def test_rectangular_fp32(mm, shape):
    announce("matmul rect", shape)
    nbR, r_out, r_in, nbL, l_out, l_in = shape
    w = workloads.monarch_matmul_rect_inputs(37, *shape, seed=11)
    y = host(mm.monarch_matmul(dev(w["x"]), dev(w["R"]), dev(w["L"])))
    assert y.shape == (37, nbL * l_out)
    assert rel_l2(y, oracle.matmul(w["x"], w["R"], w["L"])) <= TOL_F32


@pytest.mark.parametrize("b", [16, 32])
def test_bf16_inputs(mm, b):
    announce("matmul bf16 b", b)
    w = workloads.monarch_matmul_inputs(batch=130, b=b, seed=3, bf16=True)
    y = host(mm.monarch_matmul(dev(w["x"], True), dev(w["R"], True), dev(w["L"], True)))
    assert rel_l2(y, oracle.matmul(w["x"], w["R"], w["L"])) <= TOL_BF16


@pytest.mark.parametrize("batch", [1, 16, 5000, 20011])
def test_bf16_config1_shape_on_the_matrix_cores(mm, batch):
    # bf16 tensors through the fp32 MFMA kernel of config 1: one vector, one tile, many ragged tiles, more tiles
    # than waves
    announce("matmul bf16 b=16 batch", batch)
    w = workloads.monarch_matmul_inputs(batch=batch, b=16, seed=batch, bf16=True)
    y = mm.monarch_matmul(dev(w["x"], True), dev(w["R"], True), dev(w["L"], True))
    assert y.dtype == torch.bfloat16
    assert rel_l2(host(y), oracle.matmul(w["x"], w["R"], w["L"])) <= TOL_BF16


def test_bf16_identity_blocks_are_the_permutation_bit_exact(mm):
    announce("matmul bf16 identity b=16")
    eye = np.tile(np.eye(16, dtype=np.float32), (16, 1, 1))
    x = workloads.round_to_bf16(np.random.default_rng(0).standard_normal((19, 256)).astype(np.float32))
    y = host(mm.monarch_matmul(dev(x, True), dev(eye, True), dev(eye, True))).astype(np.float32)
    np.testing.assert_array_equal(y, x[:, oracle.perm(16, 256)])


@pytest.mark.parametrize("b", [4, 16])
def test_identity_blocks_are_the_permutation_bit_exact(mm, b):
    # L = R = I  =>  M = P (the involution P_(b,b^2)); multiplying by 1 and adding 0 is exact.
    announce("matmul identity b", b)
    N = b * b
    eye = np.tile(np.eye(b, dtype=np.float32), (b, 1, 1))
    x = np.random.default_rng(0).standard_normal((9, N)).astype(np.float32)
    y = mm.monarch_matmul(dev(x), dev(eye), dev(eye))
    torch.cuda.synchronize()
    sigma = oracle.perm(b, N)
    assert np.array_equal(y.cpu().numpy(), x[:, sigma])
    assert np.array_equal(mm.monarch_permutation_index(b, N).numpy(), sigma)


def test_identity_blocks_rectangular_bit_exact(mm):
    announce("matmul identity rect")
    nbR, r, nbL, l = 3, 4, 6, 2
    x = np.random.default_rng(1).standard_normal((5, 12)).astype(np.float32)
    y = mm.monarch_matmul(dev(x), dev(np.tile(np.eye(r, dtype=np.float32), (nbR, 1, 1))),
                          dev(np.tile(np.eye(l, dtype=np.float32), (nbL, 1, 1))))
    torch.cuda.synchronize()
    s1, s2, s3 = oracle.perm(r, 12), oracle.perm(nbR, 12), oracle.perm(nbL, 12)
    want = x[:, s1][:, s2][:, s3]     # (P3 P2 P1 x)[i] = x[s1[s2[s3[i]]]]
    assert np.array_equal(y.cpu().numpy(), want)


def test_large_batch_sampled(mm):
    # Steady-state size of the benchmark (2^20 vectors); the oracle checks a seeded sample of rows.
    announce("matmul c1 batch 2^20 sampled")
    w = workloads.monarch_matmul_inputs(batch=1, b=16, seed=0)
    g = torch.Generator(device="cuda").manual_seed(5)
    x = torch.randn((1 << 20, 256), device="cuda", generator=g)
    y = mm.monarch_matmul(x, dev(w["R"]), dev(w["L"]))
    rows = np.random.default_rng(5).choice(1 << 20, size=64, replace=False)
    rows = np.concatenate([rows, [0, (1 << 20) - 1]])
    xs = x[torch.from_numpy(rows).cuda()].cpu().numpy()
    got = host(y[torch.from_numpy(rows).cuda()])
    assert rel_l2(got, oracle.matmul(xs, w["R"], w["L"])) <= TOL_F32
