"""GPU parity: monarch_hyena_layer (the paper's gated-convolution layer: dense projections, short depthwise
convolutions, gated long convolution, output projection) against the oracle."""
import numpy as np
import pytest
import torch

from gpu_util import TOL_BF16, TOL_F32, announce, dev, host, rel_l2
from oracle import layer
from paper_2310_12109_amd import workloads

pytestmark = pytest.mark.gpu
KEYS = ("u", "W_in", "b_in", "k_short", "k_long", "W_out", "b_out")


@pytest.fixture(scope="module")
def mm():
    from paper_2310_12109_amd import binding
    return binding


def _run(mm, w, factors, bf16, causal=True):
    return host(mm.monarch_hyena_layer(*(dev(w[k], bf16) for k in KEYS), factors, causal=causal))


def _want(w, nfft, causal=True):
    return layer.hyena_layer(*(w[k] for k in KEYS), nfft=nfft, causal=causal)


@pytest.mark.parametrize("B,n,d,ks,factors,bias", [
    (2, 1024, 64, 3, (64, 32), True),      # the long convolution on the fused 64 x 32 kernel
    (3, 128, 48, 4, (16, 16), False),      # the fused 16 x 16 kernel, no biases, odd batch
    (2, 200, 24, 1, (20, 20), True),       # a convolution in passes through the workspace; one-tap short kernels
    (1, 64, 8, 8, (8, 16), True),          # eight taps
])
def test_fp32(mm, B, n, d, ks, factors, bias):
    announce("hyena layer fp32", B, n, d, ks, factors, bias)
    w = workloads.hyena_layer_inputs(B, n, d, ks=ks, seed=n + d, bias=bias)
    nfft = int(np.prod(factors))
    # tolerance: the dense projections accumulate d products in whatever order the GEMM library picks (fp32)
    assert rel_l2(_run(mm, w, factors, False), _want(w, nfft)) <= 5 * TOL_F32


@pytest.mark.parametrize("B,n,d,ks,factors", [(4, 1024, 128, 3, (64, 32)), (2, 8192, 32, 4, (128, 128)), (5, 128, 40, 3, (16, 16))])
def test_bf16(mm, B, n, d, ks, factors):
    announce("hyena layer bf16", B, n, d, ks, factors)
    w = workloads.hyena_layer_inputs(B, n, d, ks=ks, seed=n + d + 1, bf16=True)
    nfft = int(np.prod(factors))
    # five roundings to bf16 on the way (projections, short convolutions, the convolution's own, output)
    assert rel_l2(_run(mm, w, factors, True), _want(w, nfft)) <= 1.5 * TOL_BF16


def test_bidirectional_and_short_long_kernel(mm):
    announce("hyena layer bidirectional")
    w = workloads.hyena_layer_inputs(2, 256, 16, ks=3, klen=512, seed=5)
    assert rel_l2(_run(mm, w, (16, 32), False, causal=False), _want(w, 512, causal=False)) <= 5 * TOL_F32
    w = workloads.hyena_layer_inputs(2, 256, 16, ks=3, klen=17, seed=6)
    assert rel_l2(_run(mm, w, (16, 32), False), _want(w, 512)) <= 5 * TOL_F32


def test_argument_checks_and_empty_batch(mm):
    announce("hyena layer argument checks")
    w = workloads.hyena_layer_inputs(1, 64, 8, seed=1)
    t = [dev(w[k]) for k in KEYS]
    with pytest.raises(RuntimeError):
        mm.monarch_hyena_layer(t[0][:, :60], *t[1:], (8, 16))              # n not a multiple of 8
    y = mm.monarch_hyena_layer(t[0][:0], *t[1:], (8, 16))
    assert y.shape == (0, 64, 8)


# ---- the layer with heads ----

def _run_heads(mm, w, factors, dh, bf16, causal=True):
    return host(mm.monarch_hyena_heads_layer(*(dev(w[k], bf16) for k in KEYS), factors, dh, causal=causal))


def _want_heads(w, nfft, dh, causal=True):
    return layer.hyena_heads_layer(*(w[k] for k in KEYS), dh, nfft=nfft, causal=causal)


@pytest.mark.parametrize("B,n,d,dh,ks,factors,bias", [
    (2, 1024, 32, 4, 3, (64, 32), True),     # 16 convolutions per head on the fused 64 x 32 kernel
    (3, 128, 48, 16, 4, (16, 16), False),    # the paper's head dimension: 768 batch rows of three head channels
    (1, 200, 24, 3, 2, (20, 20), True),      # a convolution in passes through the workspace, odd head dimension
    (2, 64, 8, 8, 3, (8, 16), True),         # a single head
    (2, 64, 8, 1, 3, (8, 16), True),         # head dimension 1: the layer without heads
])
def test_heads_fp32(mm, B, n, d, dh, ks, factors, bias):
    announce("hyena layer with heads fp32", B, n, d, dh, ks, factors, bias)
    w = workloads.hyena_layer_inputs(B, n, d, ks=ks, seed=n + d + dh, bias=bias, head_dim=dh)
    nfft = int(np.prod(factors))
    assert rel_l2(_run_heads(mm, w, factors, dh, False), _want_heads(w, nfft, dh)) <= 5 * TOL_F32
    if dh == 1:
        np.testing.assert_array_equal(_run_heads(mm, w, factors, 1, False), _run(mm, w, factors, False))


# (64, 32): the fused kernel forms the outer products on its loads (full rows, short rows, an odd number of batch rows);
# (16, 16): the outer-product kernel and the library's convolution
@pytest.mark.parametrize("B,n,d,dh,ks,factors", [(2, 1024, 64, 16, 3, (64, 32)), (3, 512, 24, 4, 3, (64, 32)), (1, 1000, 9, 3, 2, (64, 32)),
                                                 (5, 128, 40, 8, 3, (16, 16))])
def test_heads_bf16(mm, B, n, d, dh, ks, factors):
    announce("hyena layer with heads bf16", B, n, d, dh, ks, factors)
    w = workloads.hyena_layer_inputs(B, n, d, ks=ks, seed=n + d + dh + 1, bf16=True, head_dim=dh)
    nfft = int(np.prod(factors))
    # the roundings of the layer without heads plus the product X2~ V~ and the convolved products, each to bf16
    assert rel_l2(_run_heads(mm, w, factors, dh, True), _want_heads(w, nfft, dh)) <= 2 * TOL_BF16


def test_heads_bidirectional(mm):
    announce("hyena layer with heads bidirectional")
    w = workloads.hyena_layer_inputs(2, 256, 16, ks=3, klen=512, seed=7, head_dim=4)
    assert rel_l2(_run_heads(mm, w, (16, 32), 4, False, causal=False), _want_heads(w, 512, 4, causal=False)) <= 5 * TOL_F32


def test_heads_argument_checks(mm):
    announce("hyena layer with heads argument checks")
    w = workloads.hyena_layer_inputs(1, 64, 8, seed=1, head_dim=4)
    t = [dev(w[k]) for k in KEYS]
    for bad in (0, 3, 65, 128):                                            # out of range or not a divisor of d
        with pytest.raises(RuntimeError):
            mm.monarch_hyena_heads_layer(*t, (8, 16), bad)
    ws = torch.empty(mm.monarch_hyena_heads_layer_workspace_bytes(1, 64, 8, 64, (8, 16), 4, torch.float32) - 16, dtype=torch.uint8,
                     device="cuda")
    with pytest.raises((RuntimeError, ValueError)):
        mm.monarch_hyena_heads_layer(*t, (8, 16), 4, ws=ws)                # workspace too small
