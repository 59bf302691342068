"""GPU parity: monarch_m2_layer (the basic M2 layer: sequence mixer, dimension mixer, skip connection, layer norm;
Sec. 3.2) against the oracle."""
import numpy as np
import pytest
import torch

from gpu_util import TOL_BF16, TOL_F32, announce, dev, host, rel_l2
from oracle import layer
from paper_2310_12109_amd import workloads

pytestmark = pytest.mark.gpu

SEQ, DIM = ("R1", "L1", "R2", "L2"), ("R3", "L3", "R4", "L4")


@pytest.fixture(scope="module")
def mm():
    from paper_2310_12109_amd import binding
    return binding


def _run(mm, w, bf16=False, act=1):
    d = lambda k: dev(w[k], bf16)
    return mm.monarch_m2_layer(d("x"), [d(k) for k in SEQ], d("n_kernel"), [d(k) for k in DIM], d("d_kernel"),
                               d("gamma"), d("beta"), eps=1e-5, act=act)


def _want(w, act="relu"):
    return layer.m2_layer(w["x"], [w[k] for k in SEQ], w["n_kernel"], [w[k] for k in DIM], w["d_kernel"],
                          w["gamma"], w["beta"], 1e-5, act)[0]


@pytest.mark.parametrize("bn,bd,B", [(16, 16, 3), (16, 16, 1), (4, 8, 5), (8, 4, 5), (16, 8, 2), (8, 16, 2), (3, 5, 4), (16, 5, 2)])
def test_fp32(mm, bn, bd, B):
    # 16 x 16: both mixers on the matrix cores (transposed loads and stores; fused skip + layer norm); mixed and
    # small block sizes: the LDS-tile kernels with the same options; d = 25: the (B, n, d) access without alignment
    announce("m2 layer fp32 bn, bd, B", bn, bd, B)
    w = workloads.m2_layer_inputs(B, bn, bd, seed=bn * 100 + bd)
    assert rel_l2(host(_run(mm, w)), _want(w)) <= TOL_F32


def test_fp32_many_tiles(mm):
    # more tiles than workgroups in both kernels: 40 sequences of 256 positions x 256 features
    announce("m2 layer fp32 16, 16, B=40")
    w = workloads.m2_layer_inputs(40, 16, 16, seed=7)
    assert rel_l2(host(_run(mm, w)), _want(w)) <= TOL_F32


def test_fp32_runs_of_neighbouring_tiles(mm):
    # 2176 tiles in the sequence mixer: enough for the launcher to hand each workgroup runs of two neighbouring
    # tiles of the (B, n, d) layout
    announce("m2 layer fp32 16, 16, B=136")
    w = workloads.m2_layer_inputs(136, 16, 16, seed=11)
    got, want = host(_run(mm, w)), _want(w)
    assert rel_l2(got, want) <= TOL_F32
    err = np.linalg.norm(got - want, axis=-1) / np.linalg.norm(want, axis=-1)
    assert err.max() <= 10 * TOL_F32      # no single row is off


@pytest.mark.parametrize("bn,bd,B,act", [(32, 32, 2, 1), (32, 16, 2, 1), (16, 32, 3, 1), (64, 32, 1, 1), (32, 64, 1, 0), (32, 5, 2, 1)])
def test_fp32_blocks_of_32_and_64(mm, bn, bd, B, act):
    # n or d = 1024, 4096: that mixer runs in place on LDS tiles on the matrix cores with the layer's options (rows along the
    # middle index of (B, n, d) in pieces of four rows; activation; skip connection and layer norm); d = 25: a tile of 16
    # rows would straddle two sequences, so the sequence mixer takes the shape-generic kernel
    announce("m2 layer fp32 bn, bd, B, act", bn, bd, B, act)
    w = workloads.m2_layer_inputs(B, bn, bd, seed=bn * 100 + bd)
    assert rel_l2(host(_run(mm, w, act=act)), _want(w, "relu" if act else "none")) <= TOL_F32


def test_bf16_blocks_of_32(mm):
    announce("m2 layer bf16 32, 32")
    w = workloads.m2_layer_inputs(2, 32, 32, seed=13, bf16=True)
    y = _run(mm, w, bf16=True)
    assert y.dtype == torch.bfloat16 and rel_l2(host(y), _want(w)) <= TOL_BF16


def test_no_activation(mm):
    announce("m2 layer fp32 no activation")
    w = workloads.m2_layer_inputs(2, 16, 16, seed=8)
    assert rel_l2(host(_run(mm, w, act=0)), _want(w, "none")) <= TOL_F32


@pytest.mark.parametrize("bn,bd", [(16, 16), (8, 4)])
def test_bf16(mm, bn, bd):
    announce("m2 layer bf16 bn, bd", bn, bd)
    w = workloads.m2_layer_inputs(3, bn, bd, seed=9, bf16=True)
    y = _run(mm, w, bf16=True)
    assert y.dtype == torch.bfloat16
    # X~ is rounded to bf16 between the two kernels and the output once more
    assert rel_l2(host(y), _want(w)) <= TOL_BF16


def test_rows_are_normalised(mm):
    announce("m2 layer normalisation")
    w = workloads.m2_layer_inputs(2, 16, 16, seed=10)
    w["gamma"], w["beta"] = np.ones(256, dtype=np.float32), np.zeros(256, dtype=np.float32)
    y = host(_run(mm, w))
    assert np.abs(y.mean(-1)).max() < 1e-5 and np.abs(y.var(-1) - 1).max() < 1e-3
