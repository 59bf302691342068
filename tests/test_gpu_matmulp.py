"""GPU parity: monarch_matmulp / monarch_matmulp_backward (general order-p Monarch product, Sec. 3.1 and the appendix
definition of the p-variate Monarch matrix) against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL_BF16, TOL_F32, announce, dev, host, rel_l2
from oracle import order3, orderp
from paper_2310_12109_amd import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mm():
    from paper_2310_12109_amd import binding
    return binding


# orders 2 to 12, blocks 2 to 16, one to eight rows per tile, ragged last tiles, more tiles than workgroups
SHAPES = [(2, 2, 5), (4, 2, 9), (16, 2, 33), (3, 3, 7), (2, 4, 5), (3, 4, 11), (4, 4, 64), (8, 4, 3), (2, 6, 19), (4, 5, 10),
          (2, 12, 3), (3, 7, 2), (4, 6, 5), (5, 5, 4), (16, 3, 6), (4, 4, 5000)]


@pytest.mark.parametrize("b,p,batch", SHAPES)
def test_forward_fp32(mm, b, p, batch):
    announce("matmulp fp32 b, p, batch", b, p, batch)
    w = workloads.monarch_matmulp_inputs(batch, b, p, seed=b + p + batch)
    assert rel_l2(host(mm.monarch_matmulp(dev(w["x"]), dev(w["B"]))), orderp.matmulp(w["x"], w["B"])) <= TOL_F32


def test_forward_is_the_order_two_and_order_three_entry_point(mm):
    announce("matmulp against matmul and matmul3")
    w = workloads.monarch_matmulp_inputs(9, 8, 3, seed=1)
    y3 = host(mm.monarch_matmul3(dev(w["x"]), dev(w["B"][0]), dev(w["B"][1]), dev(w["B"][2])))
    assert rel_l2(host(mm.monarch_matmulp(dev(w["x"]), dev(w["B"]))), y3) <= TOL_F32
    assert rel_l2(y3, order3.matmul3(w["x"], w["B"][0], w["B"][1], w["B"][2])) <= TOL_F32
    w = workloads.monarch_matmulp_inputs(9, 8, 2, seed=2)
    assert rel_l2(host(mm.monarch_matmulp(dev(w["x"]), dev(w["B"]))), oracle.matmul(w["x"], w["B"][0], w["B"][1])) <= TOL_F32


def test_identity_blocks_leave_the_vector(mm):
    # with identity blocks the factors do nothing and the two digit reversals cancel
    announce("matmulp identity blocks")
    b, p = 3, 5
    w = workloads.monarch_matmulp_inputs(4, b, p, seed=3)
    eye = np.broadcast_to(np.eye(b, dtype=np.float32), (p, b ** (p - 1), b, b)).copy()
    y = host(mm.monarch_matmulp(dev(w["x"]), dev(eye))).astype(np.float32)
    want = orderp.matmulp(w["x"], eye)
    np.testing.assert_array_equal(y, want.astype(np.float32))


@pytest.mark.parametrize("b,p", [(4, 4), (2, 8), (8, 4)])
def test_forward_bf16(mm, b, p):
    announce("matmulp bf16 b, p", b, p)
    w = workloads.monarch_matmulp_inputs(13, b, p, seed=b + p, bf16=True)
    y = mm.monarch_matmulp(dev(w["x"], True), dev(w["B"], True))
    assert y.dtype == torch.bfloat16
    assert rel_l2(host(y), orderp.matmulp(w["x"], w["B"])) <= TOL_BF16


# tiles of four rows: lone rows, ragged tails, more tiles than workgroups; every register-array size (b <= 2, 4, 8, 16)
BACK = [(2, 2, 5), (16, 2, 33), (3, 3, 7), (2, 4, 5), (3, 4, 11), (4, 4, 64), (8, 4, 3), (2, 6, 19), (4, 5, 10), (2, 12, 3), (4, 6, 2),
        (16, 3, 6), (5, 5, 1), (12, 3, 9), (7, 4, 6), (4, 4, 2500)]


@pytest.mark.parametrize("b,p,batch", BACK)
def test_backward_fp32(mm, b, p, batch):
    announce("matmulp backward fp32 b, p, batch", b, p, batch)
    w = workloads.monarch_matmulp_inputs(batch, b, p, seed=100 + b + p)
    dx, dB = mm.monarch_matmulp_backward(dev(w["x"]), dev(w["B"]), dev(w["dy"]))
    want_dx, want_dB = orderp.matmulp_backward(w["x"], w["B"], w["dy"])
    assert rel_l2(host(dx), want_dx) <= TOL_F32
    assert dB.dtype == torch.float32
    for s in range(p):
        assert rel_l2(host(dB[s]), want_dB[s]) <= TOL_F32


def test_backward_bf16_and_partial_outputs(mm):
    announce("matmulp backward bf16, partial outputs")
    w = workloads.monarch_matmulp_inputs(17, 4, 4, seed=3, bf16=True)
    want_dx, want_dB = orderp.matmulp_backward(w["x"], w["B"], w["dy"])
    dx, dB = mm.monarch_matmulp_backward(dev(w["x"], True), dev(w["B"], True), dev(w["dy"], True))
    assert dx.dtype == torch.bfloat16 and rel_l2(host(dx), want_dx) <= TOL_BF16
    assert rel_l2(host(dB), want_dB) <= TOL_F32 * 10      # fp32 sums of products of bf16 values: no bf16 rounding in them
    dx, none = mm.monarch_matmulp_backward(dev(w["x"], True), dev(w["B"], True), dev(w["dy"], True), need_dB=False)
    assert none is None and rel_l2(host(dx), want_dx) <= TOL_BF16
    none, dB = mm.monarch_matmulp_backward(dev(w["x"], True), dev(w["B"], True), dev(w["dy"], True), need_dx=False)
    assert none is None and rel_l2(host(dB), want_dB) <= TOL_F32 * 10


def test_empty_batch_and_argument_checks(mm):
    announce("matmulp empty batch, argument checks")
    w = workloads.monarch_matmulp_inputs(4, 4, 4, seed=4)
    x, B, dy = dev(w["x"]), dev(w["B"]), dev(w["dy"])
    assert mm.monarch_matmulp(x[:0], B).shape == (0, 256)
    dx, dB = mm.monarch_matmulp_backward(x[:0], B, dy[:0])
    assert dx.shape == (0, 256) and float(dB.abs().max()) == 0
    big = torch.zeros((13, 1, 2, 2), device="cuda")                       # 2^13 > 4096
    with pytest.raises(RuntimeError):
        mm.monarch_matmulp(torch.zeros((1, 8192), device="cuda"), big)
    with pytest.raises(RuntimeError):                                     # blocks of 17
        mm.monarch_matmulp(torch.zeros((1, 289), device="cuda"), torch.zeros((2, 17, 17, 17), device="cuda"))
    with pytest.raises(RuntimeError):                                     # order 1
        mm.monarch_matmulp_backward(torch.zeros((1, 4), device="cuda"), torch.zeros((1, 1, 4, 4), device="cuda"),
                                    torch.zeros((1, 4), device="cuda"))
