"""GPU parity: monarch_mixer (sequence mixer with two general order-2 Monarch matrices, Sec. 3.2 Eq. 2, gated)
against the oracle."""
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


def _run(mm, w, bf16=False):
    return mm.monarch_mixer(*(dev(w[k], bf16) for k in ("u", "K", "g_in", "g_out", "R1", "L1", "R2", "L2")))


def _want(w):
    return oracle.mixer(*(w[k] for k in ("u", "K", "g_in", "g_out", "R1", "L1", "R2", "L2")))


@pytest.mark.parametrize("B,H", [(4, 16), (1, 1), (3, 7), (5, 13), (16, 96)])
def test_n256_fp32(mm, B, H):
    # tiles of 16 rows on the matrix cores: one tile, one row, ragged tiles whose rows change channel (3 x 7,
    # 5 x 13), and 96 tiles
    announce("mixer fp32 b=16 B,H", B, H)
    w = workloads.mixer_inputs(B, H, 16, seed=B * 100 + H)
    assert rel_l2(host(_run(mm, w)), _want(w)) <= TOL_F32


@pytest.mark.parametrize("gates", [(True, False), (False, True), (False, False)])
def test_n256_fp32_gates_absent(mm, gates):
    announce("mixer fp32 b=16 gates", gates)
    w = workloads.mixer_inputs(3, 11, 16, seed=7, gates=gates)
    assert rel_l2(host(_run(mm, w)), _want(w)) <= TOL_F32


def test_n256_fp32_more_tiles_than_workgroups(mm):
    # 1251 tiles on at most 512 workgroups, the last tile ragged; the output must not depend on which workgroup
    # and which of its iterations took a tile: checked against the oracle on a sample of rows from the whole range
    B, H = 41, 488   # 20008 rows
    announce("mixer fp32 b=16 B,H", B, H)
    w = workloads.mixer_inputs(B, H, 16, seed=3)
    y = host(_run(mm, w)).reshape(B * H, 256)
    rows = np.unique(np.concatenate([np.arange(0, 40), np.arange(B * H - 40, B * H),
                                     np.random.default_rng(0).integers(0, B * H, 400)]))
    flat = {k: w[k].reshape(B * H, 256) for k in ("u", "g_in", "g_out")}
    for r in rows:
        h = r % H
        want = oracle.mixer(flat["u"][r][None, None], w["K"][h][None], flat["g_in"][r][None, None], flat["g_out"][r][None, None],
                            w["R1"], w["L1"], w["R2"], w["L2"])[0, 0]
        assert rel_l2(y[r], want) <= TOL_F32, r
    assert np.isfinite(y).all()


@pytest.mark.parametrize("b", [2, 3, 8, 32, 64])
def test_other_block_sizes_fp32(mm, b):
    announce("mixer fp32 b", b)
    w = workloads.mixer_inputs(3, 5, b, seed=b)
    assert rel_l2(host(_run(mm, w)), _want(w)) <= TOL_F32


@pytest.mark.parametrize("b,B,H,gates,bf16", [(32, 7, 5, (True, True), False), (32, 40, 13, (False, True), False),
                                              (32, 9, 4, (True, False), True), (64, 3, 7, (True, True), False),
                                              (64, 5, 9, (False, False), False), (64, 4, 6, (True, True), True)])
def test_blocks_of_32_and_64_in_place_on_the_matrix_cores(mm, b, B, H, gates, bf16):
    # ragged tiles whose rows change channel, each gate combination, fp32 and bf16 tensors
    announce("mixer in place b, B, H, gates, bf16", b, B, H, gates, bf16)
    w = workloads.mixer_inputs(B, H, b, seed=b + B + H, gates=gates, bf16=bf16)
    assert rel_l2(host(_run(mm, w, bf16)), _want(w)) <= (TOL_BF16 if bf16 else TOL_F32)


@pytest.mark.parametrize("b", [4, 16, 32])
def test_bf16(mm, b):
    announce("mixer bf16 b", b)
    w = workloads.mixer_inputs(4, 9, b, seed=b, bf16=True)
    y = _run(mm, w, bf16=True)
    assert y.dtype == torch.bfloat16
    assert rel_l2(host(y), _want(w)) <= TOL_BF16


@pytest.mark.parametrize("gates", [(True, True), (False, False), (True, False)])
def test_bf16_n256_many_tiles(mm, gates):
    # bf16 rows through the matrix-core kernel (two rows per load instruction, widened into LDS): 143 tiles, ragged
    announce("mixer bf16 b=16 many tiles, gates", gates)
    w = workloads.mixer_inputs(13, 175, 16, seed=21, gates=gates, bf16=True)
    assert rel_l2(host(_run(mm, w, bf16=True)), _want(w)) <= TOL_BF16


def test_bf16_identity_blocks_are_exact_up_to_the_output_rounding(mm):
    # identity blocks: the mixer is g_out o P(K o P(g_in o u)); fp32 products of bf16 values, one rounding at the store
    announce("mixer bf16 identity blocks")
    w = workloads.mixer_inputs(2, 5, 16, seed=22, bf16=True)
    eye = np.broadcast_to(np.eye(16, dtype=np.float32), (16, 16, 16)).copy()
    for k in ("R1", "L1", "R2", "L2"):
        w[k] = eye
    perm = oracle.perm(16, 256)
    t = ((w["g_in"] * w["u"]).astype(np.float32)[..., perm] * w["K"][None]).astype(np.float32)
    want = workloads.round_to_bf16((t[..., perm] * w["g_out"]).astype(np.float32))
    np.testing.assert_array_equal(host(_run(mm, w, bf16=True)).astype(np.float32), want)


def test_identity_blocks_reduce_to_the_gated_product(mm):
    # all four factors the identity: P P P = P for the involution P of a square Monarch matrix, so M = P and
    # y = g_out o P (K o P (g_in o u)): an index identity, exact in fp32
    announce("mixer identity blocks")
    w = workloads.mixer_inputs(2, 3, 16, seed=1)
    eye = np.broadcast_to(np.eye(16, dtype=np.float32), (16, 16, 16)).copy()
    for k in ("R1", "L1", "R2", "L2"):
        w[k] = eye
    perm = oracle.perm(16, 256)
    a = (w["g_in"] * w["u"]).astype(np.float32)
    t = (a[..., perm] * w["K"][None]).astype(np.float32)
    want = (t[..., perm] * w["g_out"]).astype(np.float32)
    np.testing.assert_array_equal(host(_run(mm, w)).astype(np.float32), want)


def test_empty_batch(mm):
    w = workloads.mixer_inputs(1, 4, 16, seed=0)
    w["u"] = w["u"][:0]; w["g_in"] = w["g_in"][:0]; w["g_out"] = w["g_out"][:0]
    assert _run(mm, w).shape == (0, 4, 256)
