"""GPU parity: monarch_matmul3 / monarch_matmul3_backward (general order-3 Monarch product, Sec. 3.1 and the
appendix definition of order-p Monarch matrices) against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL_BF16, TOL_F32, announce, dev, host, rel_l2
from oracle import order3
from paper_2310_12109_amd import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mm():
    from paper_2310_12109_amd import binding
    return binding


def _f(w, bf16=False):
    return [dev(w[k], bf16) for k in ("x", "B1", "B2", "B3")]


@pytest.mark.parametrize("b,batch", [(2, 5), (3, 7), (4, 64), (8, 19), (16, 9), (16, 1), (8, 3000)])
def test_forward_fp32(mm, b, batch):
    # one to eight rows per tile, ragged last tiles, more tiles than workgroups (b = 8, batch 3000)
    announce("matmul3 fp32 b, batch", b, batch)
    w = workloads.monarch_matmul3_inputs(batch, b, seed=b + batch)
    assert rel_l2(host(mm.monarch_matmul3(*_f(w))), order3.matmul3(w["x"], w["B1"], w["B2"], w["B3"])) <= TOL_F32


@pytest.mark.parametrize("batch", [8, 21, 2600])
def test_forward_b16_on_the_matrix_cores(mm, batch):
    # tiles of 8 rows worked in place in LDS: one tile, ragged tiles, more tiles than workgroups
    announce("matmul3 fp32 b=16 batch", batch)
    w = workloads.monarch_matmul3_inputs(batch, 16, seed=batch)
    got, want = host(mm.monarch_matmul3(*_f(w))), order3.matmul3(w["x"], w["B1"], w["B2"], w["B3"])
    assert rel_l2(got, want) <= TOL_F32
    err = np.linalg.norm(got - want, axis=-1) / np.linalg.norm(want, axis=-1)
    assert err.max() <= 10 * TOL_F32      # no single row is off


def test_forward_b16_identity_blocks_reverse_the_digits(mm):
    announce("matmul3 identity blocks b=16")
    b = 16
    w = workloads.monarch_matmul3_inputs(5, b, seed=2)
    eye = np.broadcast_to(np.eye(b, dtype=np.float32), (b * b, b, b)).copy()
    y = host(mm.monarch_matmul3(dev(w["x"]), dev(eye), dev(eye), dev(eye))).astype(np.float32)
    np.testing.assert_array_equal(y.reshape(5, b, b, b), w["x"].reshape(5, b, b, b).transpose(0, 3, 2, 1))


def test_forward_against_the_dense_matrix(mm):
    # the same product through the oracle's dense matrix (dense permutations and block-diagonals)
    announce("matmul3 fp32 dense b=4")
    w = workloads.monarch_matmul3_inputs(11, 4, seed=1)
    M = oracle.monarch3_dense(w["B1"], w["B2"], w["B3"]).real
    assert rel_l2(host(mm.monarch_matmul3(*_f(w))), w["x"].astype(np.float64) @ M.T) <= TOL_F32


@pytest.mark.parametrize("b", [4, 8, 16])
def test_forward_bf16(mm, b):
    announce("matmul3 bf16 b", b)
    w = workloads.monarch_matmul3_inputs(13, b, seed=b, bf16=True)
    y = mm.monarch_matmul3(*_f(w, True))
    assert y.dtype == torch.bfloat16
    assert rel_l2(host(y), order3.matmul3(w["x"], w["B1"], w["B2"], w["B3"])) <= TOL_BF16


def test_identity_blocks_reverse_the_digits(mm):
    announce("matmul3 identity blocks")
    b = 4
    w = workloads.monarch_matmul3_inputs(3, b, seed=2)
    eye = np.broadcast_to(np.eye(b, dtype=np.float32), (b * b, b, b)).copy()
    y = host(mm.monarch_matmul3(dev(w["x"]), dev(eye), dev(eye), dev(eye))).astype(np.float32)
    np.testing.assert_array_equal(y.reshape(3, b, b, b), w["x"].reshape(3, b, b, b).transpose(0, 3, 2, 1))


@pytest.mark.parametrize("b,batch", [(2, 5), (3, 7), (4, 64), (8, 19), (16, 5), (8, 1500)])
def test_backward_fp32(mm, b, batch):
    announce("matmul3 backward fp32 b, batch", b, batch)
    w = workloads.monarch_matmul3_inputs(batch, b, seed=100 + b)
    got = mm.monarch_matmul3_backward(*_f(w), dev(w["dy"]))
    want = order3.matmul3_backward(w["x"], w["B1"], w["B2"], w["B3"], w["dy"])
    for g, x in zip(got, want):
        assert rel_l2(host(g), x) <= TOL_F32
    assert all(g.dtype == torch.float32 for g in got[1:])


@pytest.mark.parametrize("batch", [1, 4, 9, 1030])
def test_backward_b16_on_the_matrix_cores(mm, batch):
    # tiles of four rows: a lone row, one full tile, a ragged tail, several tiles per workgroup
    announce("matmul3 backward fp32 b=16 batch", batch)
    w = workloads.monarch_matmul3_inputs(batch, 16, seed=200 + batch)
    got = mm.monarch_matmul3_backward(*_f(w), dev(w["dy"]))
    want = order3.matmul3_backward(w["x"], w["B1"], w["B2"], w["B3"], w["dy"])
    for g, x in zip(got, want):
        assert rel_l2(host(g), x) <= TOL_F32


def test_backward_b16_bf16_and_partial_outputs(mm):
    announce("matmul3 backward bf16 b=16, partial outputs")
    w = workloads.monarch_matmul3_inputs(11, 16, seed=31, bf16=True)
    want = order3.matmul3_backward(w["x"], w["B1"], w["B2"], w["B3"], w["dy"])
    got = mm.monarch_matmul3_backward(*_f(w, True), dev(w["dy"], True))
    assert got[0].dtype == torch.bfloat16 and rel_l2(host(got[0]), want[0]) <= TOL_BF16
    for g, x in zip(got[1:], want[1:]):
        assert rel_l2(host(g), x) <= TOL_F32 * 10
    dx, d1, d2, d3 = mm.monarch_matmul3_backward(*_f(w, True), dev(w["dy"], True), need_dB=False)
    assert d1 is None and d2 is None and d3 is None and rel_l2(host(dx), want[0]) <= TOL_BF16


def test_backward_bf16(mm):
    announce("matmul3 backward bf16 b=8")
    w = workloads.monarch_matmul3_inputs(17, 8, seed=3, bf16=True)
    got = mm.monarch_matmul3_backward(*_f(w, True), dev(w["dy"], True))
    want = order3.matmul3_backward(w["x"], w["B1"], w["B2"], w["B3"], w["dy"])
    assert got[0].dtype == torch.bfloat16 and rel_l2(host(got[0]), want[0]) <= TOL_BF16
    for g, x in zip(got[1:], want[1:]):
        assert rel_l2(host(g), x) <= TOL_F32 * 10    # fp32 sums of products of bf16 values: no bf16 rounding in them


def test_backward_partial_outputs_and_empty_batch(mm):
    announce("matmul3 backward partial outputs")
    w = workloads.monarch_matmul3_inputs(6, 4, seed=4)
    dx, d1, d2, d3 = mm.monarch_matmul3_backward(*_f(w), dev(w["dy"]), need_dB=False)
    assert d1 is None and d3 is None
    assert rel_l2(host(dx), order3.matmul3_backward(w["x"], w["B1"], w["B2"], w["B3"], w["dy"])[0]) <= TOL_F32
    w0 = {k: (v[:0] if k in ("x", "dy") else v) for k, v in w.items()}
    dx, d1, d2, d3 = mm.monarch_matmul3_backward(*_f(w0), dev(w0["dy"]))
    assert dx.shape == (0, 64) and float(d1.abs().max()) == 0 and float(d3.abs().max()) == 0
    assert mm.monarch_matmul3(*_f(w0)).shape == (0, 64)
