"""Helpers shared by the GPU parity tests (marshalling and error metrics only)."""
import numpy as np
import torch

TOL_F32 = 1e-5    # relative L2, fp32 paths
TOL_BF16 = 2e-2   # relative L2, bf16-in / fp32-accumulate paths


def dev(a, bf16=False):
    """numpy float32 array -> device tensor; bf16 arrays are already bf16-representable."""
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if bf16 else t


def host(t):
    torch.cuda.synchronize()
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel_l2(got, want):
    got = np.asarray(got)
    want = np.asarray(want)
    dt = np.complex128 if (np.iscomplexobj(got) or np.iscomplexobj(want)) else np.float64
    got, want = got.astype(dt), want.astype(dt)
    denom = np.linalg.norm(want.ravel())
    err = np.linalg.norm((got - want).ravel())
    return err / denom if denom > 0 else err


def announce(*parts):
    """Print what is about to run on the GPU, flushed, so a fault can be attributed."""
    print("[gpu-case]", *parts, flush=True)
