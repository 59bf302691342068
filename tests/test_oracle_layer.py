"""Pins for the oracle's basic M2 layer (sequence mixer, dimension mixer, skip connection, layer norm)."""
import numpy as np
import pytest
import torch

import oracle
from oracle import layer
from paper_2310_12109_amd import workloads


def _args(w):
    return (w["x"], tuple(w[k] for k in ("R1", "L1", "R2", "L2")), w["n_kernel"],
            tuple(w[k] for k in ("R3", "L3", "R4", "L4")), w["d_kernel"], w["gamma"], w["beta"])


@pytest.mark.parametrize("bn,bd", [(2, 3), (4, 4), (3, 5)])
def test_without_activation_the_mixers_are_the_c_oracles_mixer(bn, bd):
    # act = none: X~ is the sequence mixer of the C oracle on the transposed input, and the pre-norm output the
    # same mixer along the features with one shared kernel row
    w = workloads.m2_layer_inputs(3, bn, bd, seed=bn * 10 + bd)
    out, xtil = layer.m2_layer(*_args(w), act="none")
    B, n, d = w["x"].shape
    xt = np.ascontiguousarray(w["x"].transpose(0, 2, 1))
    want = oracle.mixer(xt, w["n_kernel"], None, None, w["R1"], w["L1"], w["R2"], w["L2"]).transpose(0, 2, 1)
    assert np.abs(xtil - want).max() < 1e-10
    y = oracle.mixer(np.ascontiguousarray(xtil).reshape(B * n, 1, d), w["d_kernel"][None], None, None,
                     w["R3"], w["L3"], w["R4"], w["L4"]).reshape(B, n, d)
    ln = torch.nn.functional.layer_norm(torch.from_numpy(y + xtil), (d,), torch.from_numpy(w["gamma"].astype(np.float64)),
                                        torch.from_numpy(w["beta"].astype(np.float64)), 1e-5).numpy()
    assert np.abs(out - ln).max() < 1e-10


def test_identity_blocks_reduce_to_index_operations():
    # all eight factors the identity: every Monarch matrix is the permutation P, and the layer is
    # X~ = (P relu(K o P X^T))^T, Y = P relu(k o P X~): gathers, products and maxima only
    bn, bd = 3, 4
    w = workloads.m2_layer_inputs(2, bn, bd, seed=1)
    for k, b in (("R1", bn), ("L1", bn), ("R2", bn), ("L2", bn), ("R3", bd), ("L3", bd), ("R4", bd), ("L4", bd)):
        w[k] = np.broadcast_to(np.eye(b), (b, b, b)).copy()
    out, xtil = layer.m2_layer(*_args(w))
    pn, pd = oracle.perm(bn, bn * bn), oracle.perm(bd, bd * bd)
    x = w["x"].astype(np.float64)
    xt = x.transpose(0, 2, 1)
    want = np.maximum(xt[..., pn] * w["n_kernel"][None], 0)[..., pn].transpose(0, 2, 1)
    assert np.abs(xtil - want).max() < 1e-12
    r = np.maximum(want[..., pd] * w["d_kernel"][None, None], 0)[..., pd] + want
    ln = torch.nn.functional.layer_norm(torch.from_numpy(r), (bd * bd,), torch.from_numpy(w["gamma"].astype(np.float64)),
                                        torch.from_numpy(w["beta"].astype(np.float64)), 1e-5).numpy()
    assert np.abs(out - ln).max() < 1e-10


def test_the_activation_sits_between_the_kernel_product_and_the_second_matrix():
    # with a kernel of -1 everywhere and M1 x >= 0 the activation zeroes everything: X~ = 0 and the output is the
    # layer-norm bias; had the activation been applied before the kernel product it would not be
    bn, bd = 2, 2
    w = workloads.m2_layer_inputs(1, bn, bd, seed=2)
    for k in ("R1", "L1", "R2", "L2"):
        w[k] = np.abs(w[k])
    w["x"] = np.abs(w["x"])
    w["n_kernel"] = -np.ones_like(w["n_kernel"])
    out, xtil = layer.m2_layer(*_args(w))
    assert np.abs(xtil).max() == 0
    assert np.abs(out - w["beta"][None, None]).max() < 1e-6    # (0 - 0) / sqrt(eps) * gamma + beta


def test_layer_norm_statistics():
    w = workloads.m2_layer_inputs(2, 4, 4, seed=3)
    w["gamma"], w["beta"] = np.ones(16), np.zeros(16)
    out, _ = layer.m2_layer(*_args(w))
    assert np.abs(out.mean(-1)).max() < 1e-12
    assert np.abs(out.var(-1) - 1).max() < 1e-3       # 1 / (1 + eps / var)
