"""Seeded synthetic inputs shaped like the paper's workloads.

Only input generation lives here (random draws, decay envelopes, the dense
gate projections that sit *outside* the Monarch hot path, bf16 rounding of
inputs).  Nothing of the method's arithmetic: both the CPU oracle's tests and
the GPU path's tests/benchmark consume these arrays unchanged.

All generators return float32 numpy arrays; with ``bf16=True`` every array is
first rounded to the nearest bf16 value (ties to even) so that the GPU path
(which stores bf16) and the oracle (which reads the float32 array) see exactly
the same numbers.
"""
import numpy as np


def round_to_bf16(a):
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((x >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((x + bias) & np.uint32(0xFFFF0000)).view(np.float32)


def _finish(d, bf16):
    if not bf16:
        return {k: (np.ascontiguousarray(v, dtype=np.float32) if isinstance(v, np.ndarray) else v)
                for k, v in d.items()}
    return {k: (round_to_bf16(v) if isinstance(v, np.ndarray) else v) for k, v in d.items()}


def monarch_matmul_inputs(batch=64, b=16, seed=0, bf16=False):
    """Config 1: square order-2 Monarch, N = b*b; L, R ~ N(0, 1/b), x ~ N(0, 1)."""
    rng = np.random.default_rng(seed)
    N = b * b
    x = rng.standard_normal((batch, N))
    R = rng.standard_normal((b, b, b)) / np.sqrt(b)
    L = rng.standard_normal((b, b, b)) / np.sqrt(b)
    return _finish({"x": x, "R": R, "L": L}, bf16)


def monarch_matmul_rect_inputs(batch, nbR, r_out, r_in, nbL, l_out, l_in, seed=0, bf16=False):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((batch, nbR * r_in))
    R = rng.standard_normal((nbR, r_out, r_in)) / np.sqrt(r_in)
    L = rng.standard_normal((nbL, l_out, l_in)) / np.sqrt(l_in)
    return _finish({"x": x, "R": R, "L": L}, bf16)


def monarch_matmul3_inputs(batch, b, seed=0, bf16=False):
    """General order-3 Monarch product, N = b^3: x, dy ~ N(0, 1); three factors of b*b blocks ~ N(0, 1/b)."""
    rng = np.random.default_rng(seed)
    d = {"x": rng.standard_normal((batch, b ** 3)), "dy": rng.standard_normal((batch, b ** 3))}
    for name in ("B1", "B2", "B3"):
        d[name] = rng.standard_normal((b * b, b, b)) / np.sqrt(b)
    return _finish(d, bf16)


def monarch_matmulp_inputs(batch, b, p, seed=0, bf16=False):
    """General order-p Monarch product, N = b^p: x, dy ~ N(0, 1); the p factors B: (p, b^(p-1), b, b) ~ N(0, 1/b)."""
    rng = np.random.default_rng(seed)
    d = {"x": rng.standard_normal((batch, b ** p)), "dy": rng.standard_normal((batch, b ** p)),
         "B": rng.standard_normal((p, b ** (p - 1), b, b)) / np.sqrt(b)}
    return _finish(d, bf16)


def m2_layer_inputs(B, bn, bd, seed=0, bf16=False):
    """Basic M2 layer: x ~ N(0, 1) of shape (B, n, d), n = bn^2, d = bd^2; eight factors ~ N(0, 1/block size);
    kernels n_kernel (d, n), d_kernel (d,) ~ N(0, 1); layer-norm weight 1 + N(0, 0.1^2), bias N(0, 0.1^2)."""
    rng = np.random.default_rng(seed)
    n, d = bn * bn, bd * bd
    w = {"x": rng.standard_normal((B, n, d)), "n_kernel": rng.standard_normal((d, n)), "d_kernel": rng.standard_normal(d),
         "gamma": 1.0 + 0.1 * rng.standard_normal(d), "beta": 0.1 * rng.standard_normal(d)}
    for name in ("R1", "L1", "R2", "L2"):
        w[name] = rng.standard_normal((bn, bn, bn)) / np.sqrt(bn)
    for name in ("R3", "L3", "R4", "L4"):
        w[name] = rng.standard_normal((bd, bd, bd)) / np.sqrt(bd)
    return _finish(w, bf16)


def mixer_inputs(B, H, b, seed=0, gates=(True, True), bf16=False):
    """Learned-Monarch sequence mixer: u, gates ~ N(0, 1) of shape (B, H, b*b), kernel K ~ N(0, 1) of shape
    (H, b*b) in the transform domain, four factors ~ N(0, 1/b) of shape (b, b, b)."""
    rng = np.random.default_rng(seed)
    N = b * b
    d = {"u": rng.standard_normal((B, H, N)), "K": rng.standard_normal((H, N))}
    d["g_in"] = rng.standard_normal((B, H, N)) if gates[0] else None
    d["g_out"] = rng.standard_normal((B, H, N)) if gates[1] else None
    for name in ("R1", "L1", "R2", "L2"):
        d[name] = rng.standard_normal((b, b, b)) / np.sqrt(b)
    return _finish(d, bf16)


def hyena_layer_inputs(B, n, d, ks=3, klen=None, seed=0, bias=True, bf16=False, head_dim=1):
    """Gated-convolution layer (projections, short and long convolutions): u ~ N(0, 1) of shape (B, n, d), the
    projection matrices ~ N(0, 1/d) (W_in: (3d, d), W_out: (d, d)), biases ~ N(0, 0.1^2), short kernels
    ~ N(0, 1/ks) of shape (3d, ks), the long kernel (d / head_dim, klen) ~ N(0, 1) exp(-0.01 t) (one row per head)."""
    rng = np.random.default_rng(seed)
    klen = n if klen is None else klen
    w = {"u": rng.standard_normal((B, n, d)), "W_in": rng.standard_normal((3 * d, d)) / np.sqrt(d),
         "W_out": rng.standard_normal((d, d)) / np.sqrt(d), "k_short": rng.standard_normal((3 * d, ks)) / np.sqrt(ks),
         "k_long": rng.standard_normal((d // head_dim, klen)) * np.exp(-0.01 * np.arange(klen))[None, :]}
    w["b_in"] = 0.1 * rng.standard_normal(3 * d) if bias else None
    w["b_out"] = 0.1 * rng.standard_normal(d) if bias else None
    return _finish(w, bf16)


def blocky_inputs(B, H, n, b, seed=0, noise=0.05, klen=None, gates=True, bf16=False):
    """Polynomial-parameterised Monarch convolution: coefficient matrices Lt, Rt (b*b, b) = the pattern that gives
    the DFT (identity in every block of Rt and in the top block of Lt) plus N(0, noise^2) everywhere, a learned
    perturbation of the Fourier transform; u, gates ~ N(0, 1) of shape (B, H, n); k (H, klen) with a decaying
    envelope.  Parameters (Lt, Rt, k) stay float32; with bf16=True only u and the gates are rounded to bf16."""
    rng = np.random.default_rng(seed)
    N = b * b
    klen = n if klen is None else klen
    Lt = noise * rng.standard_normal((N, b))
    Lt[:b, :] += np.eye(b)
    Rt = noise * rng.standard_normal((N, b)) + np.tile(np.eye(b), (b, 1))
    k = rng.standard_normal((H, klen)) * np.exp(-0.05 * np.arange(klen))[None, :]
    par = _finish({"Lt": Lt, "Rt": Rt, "k": k}, False)
    act = {"u": rng.standard_normal((B, H, n))}
    act["g_in"] = rng.standard_normal((B, H, n)) if gates else None
    act["g_out"] = rng.standard_normal((B, H, n)) if gates else None
    par.update(_finish(act, bf16))
    return par


def decaying_kernel(rng, H, klen, rate=0.01, two_sided=False, nfft=None):
    """k[h,t] = N(0,1) * exp(-rate*t).  two_sided: length nfft, lag -l stored at nfft-l."""
    if not two_sided:
        t = np.arange(klen)
        return rng.standard_normal((H, klen)) * np.exp(-rate * t)[None, :]
    lag = np.arange(nfft)
    dist = np.minimum(lag, nfft - lag)
    return rng.standard_normal((H, nfft)) * np.exp(-rate * dist)[None, :]


def conv_inputs(B, H, n, seed, gates="projected", bf16=False, two_sided_nfft=None):
    """Configs 2-5: u ~ N(0,1); k decaying Gaussian; gates either dense projections
    of u over the channel axis with W ~ N(0, 1/H) (config 2) or plain N(0,1)."""
    rng = np.random.default_rng(seed)
    u = rng.standard_normal((B, H, n)).astype(np.float32)
    if two_sided_nfft:
        k = decaying_kernel(rng, H, two_sided_nfft, two_sided=True, nfft=two_sided_nfft)
    else:
        k = decaying_kernel(rng, H, n)
    if gates == "projected":
        W1 = (rng.standard_normal((H, H)) / np.sqrt(H)).astype(np.float32)
        W2 = (rng.standard_normal((H, H)) / np.sqrt(H)).astype(np.float32)
        g_in = np.matmul(W1.T[None], u)      # g[b,:,t] = W^T u[b,:,t]: a dense projection over channels
        g_out = np.matmul(W2.T[None], u)
    elif gates == "normal":
        g_in = rng.standard_normal((B, H, n)).astype(np.float32)
        g_out = rng.standard_normal((B, H, n)).astype(np.float32)
    else:
        g_in = g_out = None
    return _finish({"u": u, "k": k, "g_in": g_in, "g_out": g_out}, bf16)


def mlp_inputs(tokens, d, d_hidden, nb, order, seed, bf16=True, std=0.02, bias=True):
    """Configs 3b / 5b: x ~ N(0,1), weights ~ N(0, std^2); order-2 layers use d_mid = d."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((tokens, d)).astype(np.float32)
    out = {"x": x}
    if order == 1:
        out["W1_R"] = rng.standard_normal((nb, d_hidden // nb, d // nb)) * std
        out["W2_R"] = rng.standard_normal((nb, d // nb, d_hidden // nb)) * std
        out["W1_L"] = out["W2_L"] = None
    else:
        out["W1_R"] = rng.standard_normal((nb, d // nb, d // nb)) * std
        out["W1_L"] = rng.standard_normal((nb, d_hidden // nb, d // nb)) * std
        out["W2_R"] = rng.standard_normal((nb, d // nb, d_hidden // nb)) * std
        out["W2_L"] = rng.standard_normal((nb, d // nb, d // nb)) * std
    out["b1"] = rng.standard_normal(d_hidden) * std if bias else None
    out["b2"] = rng.standard_normal(d) * std if bias else None
    return _finish(out, bf16)


# The five named configurations (shapes only; tensors come from the functions above).
CONFIGS = {
    "c1_matmul": dict(batch=64, b=16, seed=0),
    "c2_conv": dict(B=8, H=768, n=1024, nfft=2048, factors=(64, 32), seed=1, gates="projected"),
    "c3a_conv": dict(B=32, H=768, n=128, nfft=256, factors=(16, 16), seed=2, gates="normal"),
    "c3b_mlp": dict(tokens=32 * 128, d=768, d_hidden=3072, nb=4, seed=2),
    "c4_conv": dict(B=4, H=768, n=8192, nfft=16384, factors=(128, 128), seed=3, gates="projected"),
    "c5a_conv": dict(B=1, H=256, n=131072, nfft=262144, factors=(64, 64, 64), seed=4, gates="normal"),
    "c5b_mlp": dict(tokens=65536, d=1024, d_hidden=4096, nb=16, seed=4),
}
