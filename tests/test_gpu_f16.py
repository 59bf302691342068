"""GPU parity of the fp16 I/O type (MONARCH_F16) of the hot-path entry points against the oracle: fp16 tensors,
fp32 accumulation, tolerance of the 16-bit paths."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL_BF16, announce, host, rel_l2
from paper_2310_12109_amd import workloads

pytestmark = pytest.mark.gpu
TOL_F16 = TOL_BF16      # the bar the benchmark spec sets for 16-bit inputs with fp32 accumulation


@pytest.fixture(scope="module")
def mm():
    from paper_2310_12109_amd import binding
    return binding


def r16(a):
    """Round to the nearest fp16 value; the result stays float32 so that the oracle reads what the GPU stores."""
    return None if a is None else np.asarray(a, dtype=np.float32).astype(np.float16).astype(np.float32)


def d16(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda().to(torch.float16)


@pytest.mark.parametrize("shape", [(64, 16, 16, 16, 16, 16, 16), (37, 4, 6, 8, 3, 10, 8)])
def test_matmul_f16(mm, shape):
    announce("matmul f16", shape)
    batch, nbR, r_out, r_in, nbL, l_out, l_in = shape
    w = {k: r16(v) for k, v in workloads.monarch_matmul_rect_inputs(batch, nbR, r_out, r_in, nbL, l_out, l_in, seed=3).items()}
    y = host(mm.monarch_matmul(d16(w["x"]), d16(w["R"]), d16(w["L"])))
    assert rel_l2(y, oracle.matmul(w["x"], w["R"], w["L"])) <= TOL_F16


@pytest.mark.parametrize("factors", [(16, 16), (8, 4, 8)])
def test_fft_and_ifft_f16(mm, factors):
    announce("fft / ifft f16", factors)
    N = int(np.prod(factors))
    rng = np.random.default_rng(N)
    x = r16(rng.standard_normal((3, N)))
    X = host(mm.monarch_fft(d16(x), factors, True))
    X = X[..., 0] + 1j * X[..., 1]
    assert rel_l2(X, oracle.dft(x.astype(np.float64))) <= TOL_F16
    Xr, Xi = rng.standard_normal((2, 3, N)).astype(np.float32)
    back = host(mm.monarch_ifft(torch.from_numpy(np.stack([Xr, Xi], -1)).cuda(), factors, True, dtype=torch.float16))
    assert rel_l2(back, oracle.idft(Xr.astype(np.float64) + 1j * Xi).real) <= TOL_F16


@pytest.mark.parametrize("B,H,n,klen,factors", [
    (3, 5, 100, 37, (16, 16)),
    (2, 3, 500, 500, (8, 8, 16)),
    (5, 6, 1024, 1024, (64, 32)),     # the fused 64 x 32 kernel in fp16
    (9, 4, 1000, 504, (64, 32)),      # short rows, several batch groups
    (2, 3, 1024, 1024, (32, 64)),
])
def test_causal_conv_f16(mm, B, H, n, klen, factors):
    announce("conv f16", B, H, n, klen, factors)
    w = workloads.conv_inputs(B, H, n, seed=B + n + klen, gates="normal")
    w = {k: r16(v) for k, v in w.items()}
    w["k"] = np.ascontiguousarray(w["k"][:, :klen])
    y = host(mm.monarch_causal_conv(d16(w["u"]), d16(w["k"]), d16(w["g_in"]), d16(w["g_out"]), factors))
    want = oracle.causal_conv(w["u"], w["k"], w["g_in"], w["g_out"], nfft=int(np.prod(factors)))
    assert rel_l2(y, want) <= TOL_F16
    num = np.linalg.norm((y - want).reshape(-1, n), axis=1)
    assert (num / np.linalg.norm(want.reshape(-1, n), axis=1)).max() <= 2.5 * TOL_F16


def test_causal_conv_f16_without_gates(mm):
    announce("conv f16 no gates 64x32")
    w = {k: r16(v) for k, v in workloads.conv_inputs(4, 3, 1024, seed=12, gates="none").items()}
    y = host(mm.monarch_causal_conv(d16(w["u"]), d16(w["k"]), None, None, (64, 32)))
    assert rel_l2(y, oracle.causal_conv(w["u"], w["k"], None, None, nfft=2048)) <= TOL_F16


@pytest.mark.parametrize("order", [1, 2])
@pytest.mark.parametrize("tokens,d,dh,nb", [(37, 24, 96, 4),            # generic kernels
                                            (300, 256, 1024, 4),         # matrix-core kernel, few tokens
                                            (2100, 128, 512, 4),         # weights resident in LDS
                                            (16500, 384, 768, 4)])       # weights streamed, wide token tiles
def test_mlp_f16(mm, order, tokens, d, dh, nb):
    announce("mlp f16", order, tokens, d, dh, nb)
    w = workloads.mlp_inputs(tokens, d, dh, nb, order, seed=tokens, bf16=False, std=0.08)
    w = {k: r16(v) for k, v in w.items()}
    t = {k: d16(w[k]) for k in ("W1_R", "W1_L", "b1", "W2_R", "W2_L", "b2")}
    y = host(mm.monarch_mlp(d16(w["x"]), t["W1_R"], t["W1_L"], t["b1"], t["W2_R"], t["W2_L"], t["b2"], nb, order, 2, dh))
    want = oracle.mlp(w["x"], w["W1_R"], w["W1_L"], w["b1"], w["W2_R"], w["W2_L"], w["b2"], nb=nb, order=order, act=2)
    assert rel_l2(y, want) <= TOL_F16


def test_entry_points_outside_the_hot_path_refuse_f16(mm):
    announce("f16 refused by the widening entry points")
    u = torch.zeros((1, 2, 256), device="cuda", dtype=torch.float16)
    f = [torch.zeros((16, 16, 16), device="cuda", dtype=torch.float16) for _ in range(4)]
    with pytest.raises(mm.MonarchError) as e:
        mm.monarch_mixer(u, torch.zeros((2, 256), device="cuda", dtype=torch.float16), None, None, *f)
    assert e.value.code == mm.EDTYPE
