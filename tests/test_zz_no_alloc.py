"""GPU: monarch_causal_conv_static (the entry point that allocates nothing; its scratch is a static device array
inside the library) gives what monarch_causal_conv gives with a caller's workspace, on calls in a row that share
the array, the later ones smaller than the first."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL_BF16, TOL_F32, announce, dev, host, rel_l2
from paper_2310_12109_amd import workloads

pytestmark = pytest.mark.gpu


def _static_call(lib, t, y, factors, causal=1):
    """Straight through the C ABI: pointers and sizes only."""
    B, H, n = t["u"].shape
    f = (ctypes.c_int * len(factors))(*factors)
    ptr = lambda a: None if a is None else a.data_ptr()
    return lib.monarch_causal_conv_static(ptr(t["u"]), ptr(t["k"]), ptr(t["g_in"]), ptr(t["g_out"]), y.data_ptr(),
                                          B, H, n, t["k"].shape[1], int(np.prod(factors)), f, len(factors), causal,
                                          1 if t["u"].dtype == torch.bfloat16 else 0,
                                          torch.cuda.current_stream().cuda_stream)


@pytest.mark.parametrize("bf16,factors,shapes", [
    (True, (128, 64), [(4, 8, 4096), (2, 3, 2048), (1, 2, 1000)]),       # LDS-chunk path: spectrum of k in scratch
    (False, (32, 64), [(5, 7, 1000), (2, 3, 512)]),                      # fp32 matrix-core passes: row buffers + k_f
    (True, (16, 16, 32), [(3, 6, 4096), (1, 4, 1500)]),                  # three factors
    (False, (10, 12), [(3, 4, 50), (1, 1, 7)]),                          # generic fp32 passes
])
def test_static_scratch_calls_in_a_row_match_the_workspace_entry_point(bf16, factors, shapes):
    from paper_2310_12109_amd import binding
    lib = binding.raw()
    tol = TOL_BF16 if bf16 else TOL_F32
    for (B, H, n) in shapes:
        announce("conv static", "bf16" if bf16 else "fp32", factors, B, H, n)
        w = workloads.conv_inputs(B, H, n, seed=B + H + n, gates="normal", bf16=bf16)
        t = {k: dev(v, bf16) for k, v in w.items()}
        assert binding.monarch_causal_conv_workspace_bytes(B, H, n, n, factors, binding.BF16 if bf16 else binding.F32) > 0
        want = binding.monarch_causal_conv(t["u"], t["k"], t["g_in"], t["g_out"], factors)
        y = torch.full_like(want, float("nan"))
        rc = _static_call(lib, t, y, factors)
        assert rc == 0, lib.monarch_last_error()
        torch.cuda.synchronize()
        assert torch.equal(y, want)            # same kernels, same order of operations: identical bits
        ref = oracle.causal_conv(w["u"], w["k"], w["g_in"], w["g_out"], nfft=int(np.prod(factors)))
        assert rel_l2(host(y), ref) <= tol


def test_static_scratch_fused_shape_and_size_limit():
    from paper_2310_12109_amd import binding
    lib = binding.raw()
    announce("conv static fused shape / limit")
    # a fused shape needs no scratch at all and goes through the same entry point
    w = workloads.conv_inputs(3, 4, 1024, seed=9, gates="normal", bf16=True)
    t = {k: dev(v, True) for k, v in w.items()}
    want = binding.monarch_causal_conv(t["u"], t["k"], t["g_in"], t["g_out"], (64, 32))
    y = torch.empty_like(want)
    assert _static_call(lib, t, y, (64, 32)) == 0
    torch.cuda.synchronize()
    assert torch.equal(y, want)
    # beyond the static array: a clear error and no device work (the output stays untouched)
    B, H, n, factors = 1, 512, 16384, (32, 32, 32)
    big = {"u": torch.zeros((B, H, n), device="cuda", dtype=torch.bfloat16), "k": torch.zeros((H, n), device="cuda", dtype=torch.bfloat16),
           "g_in": None, "g_out": None}
    assert binding.monarch_causal_conv_workspace_bytes(B, H, n, n, factors, binding.BF16) > binding.STATIC_SCRATCH_BYTES
    yb = torch.full((B, H, n), 3.0, device="cuda", dtype=torch.bfloat16)
    rc = _static_call(lib, big, yb, factors)
    assert rc == binding.EWORKSPACE
    assert b"static" in lib.monarch_last_error()
    torch.cuda.synchronize()
    assert float(yb.min()) == 3.0 and float(yb.max()) == 3.0
