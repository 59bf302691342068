"""Thin ctypes binding of libmonarch.so: same names as the C ABI, argument marshalling only.

Tensors are torch CUDA(ROCm) tensors used purely as device memory; every step of the
computation runs inside the library's HIP kernels on torch's current stream.  There is no
fallback: if the library is missing, importing this module raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmonarch.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
        "(or python paper_2310_12109_amd/build.py) first; there is no fallback path")

_lib = ctypes.CDLL(LIB_PATH)

F32, BF16, F16 = 0, 1, 2
OK, EINVAL, ESHAPE, EDTYPE, EWORKSPACE, EHIP = 0, -1, -2, -3, -4, -5

_vp, _i, _i64, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t
_ip = ctypes.POINTER(ctypes.c_int)

_lib.monarch_strerror.restype = ctypes.c_char_p
_lib.monarch_strerror.argtypes = [_i]
_lib.monarch_last_error.restype = ctypes.c_char_p
_lib.monarch_permutation_index.argtypes = [_i, _i, _vp]
_lib.monarch_matmul.argtypes = [_vp, _vp, _vp, _vp, _i64, _i, _i, _i, _i, _i, _i, _i, _vp, _sz, _vp]
_lib.monarch_matmul_workspace_bytes.restype = _sz
_lib.monarch_matmul_workspace_bytes.argtypes = [_i64, _i, _i, _i, _i, _i, _i, _i]
_lib.monarch_matmul_backward.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _i, _i, _i, _i, _i, _i, _i, _vp, _sz, _vp]
_lib.monarch_matmul_backward_workspace_bytes.restype = _sz
_lib.monarch_matmul_backward_workspace_bytes.argtypes = [_i64, _i, _i, _i, _i, _i, _i, _i]
_lib.monarch_matmul3.argtypes = [_vp] * 5 + [_i64, _i, _i, _vp]
_lib.monarch_matmul3_backward.argtypes = [_vp] * 9 + [_i64, _i, _i, _vp]
_lib.monarch_matmulp.argtypes = [_vp] * 3 + [_i64, _i, _i, _i, _vp]
_lib.monarch_matmulp_backward.argtypes = [_vp] * 5 + [_i64, _i, _i, _i, _vp]
_lib.monarch_mixer_backward.argtypes = [_vp] * 17 + [_i64, _i, _i, _i, _vp, _sz, _vp]
_lib.monarch_mixer_backward_workspace_bytes.restype = _sz
_lib.monarch_mixer_backward_workspace_bytes.argtypes = [_i64, _i, _i, _i]
_lib.monarch_m2_layer.argtypes = [_vp, _vp, _i64, _i, _i] + [_vp] * 12 + [ctypes.c_float, _i, _i, _vp, _sz, _vp]
_lib.monarch_m2_layer_workspace_bytes.restype = _sz
_lib.monarch_m2_layer_workspace_bytes.argtypes = [_i64, _i, _i, _i]
_lib.monarch_hyena_layer.argtypes = [_vp] * 8 + [_i] * 6 + [_vp, _i, _i, _i, _vp, _sz, _vp]
_lib.monarch_hyena_layer_workspace_bytes.restype = _sz
_lib.monarch_hyena_layer_workspace_bytes.argtypes = [_i, _i, _i, _i, _i, _vp, _i, _i]
_lib.monarch_hyena_heads_layer.argtypes = [_vp] * 8 + [_i] * 6 + [_vp, _i, _i, _i, _i, _vp, _sz, _vp]
_lib.monarch_hyena_heads_layer_workspace_bytes.restype = _sz
_lib.monarch_hyena_heads_layer_workspace_bytes.argtypes = [_i, _i, _i, _i, _i, _vp, _i, _i, _i]
_lib.monarch_mixer.argtypes = [_vp] * 9 + [_i64, _i, _i, _i, _vp, _sz, _vp]
_lib.monarch_mixer_workspace_bytes.restype = _sz
_lib.monarch_mixer_workspace_bytes.argtypes = [_i64, _i, _i, _i]
_lib.monarch_blocky_state_bytes.restype = _sz
_lib.monarch_blocky_state_bytes.argtypes = [_i, _i]
_lib.monarch_blocky_state_offsets.argtypes = [_i, _i, ctypes.POINTER(ctypes.c_size_t)]
_lib.monarch_blocky_prepare.argtypes = [_vp, _vp, _vp, _i, _i, _i, _i, _vp, _sz, _vp]
_lib.monarch_blocky_conv.argtypes = [_vp, _vp, _vp, _vp, _sz, _vp, _i64, _i, _i, _i, _i, _vp]
_lib.monarch_fft.argtypes = [_vp, _vp, _i64, _i, _ip, _i, _i, _i, _vp, _sz, _vp]
_lib.monarch_ifft.argtypes = [_vp, _vp, _i64, _i, _ip, _i, _i, _i, _vp, _sz, _vp]
_lib.monarch_fft_workspace_bytes.restype = _sz
_lib.monarch_fft_workspace_bytes.argtypes = [_i64, _i, _ip, _i, _i]
_lib.monarch_causal_conv.argtypes = [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _ip, _i, _i, _i, _vp, _sz, _vp]
_lib.monarch_causal_conv_static.argtypes = [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _ip, _i, _i, _i, _vp]
_lib.monarch_causal_conv_workspace_bytes.restype = _sz
_lib.monarch_causal_conv_workspace_bytes.argtypes = [_i, _i, _i, _i, _i, _ip, _i, _i]
_lib.monarch_mlp.argtypes = [_vp, _vp, _i64, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _vp, _sz, _vp]
_lib.monarch_mlp_workspace_bytes.restype = _sz
_lib.monarch_mlp_workspace_bytes.argtypes = [_i64, _i, _i, _i, _i, _i, _i, _i]

EXPORTS = [
    "monarch_strerror", "monarch_last_error", "monarch_permutation_index",
    "monarch_matmul", "monarch_matmul_workspace_bytes",
    "monarch_matmul_backward", "monarch_matmul_backward_workspace_bytes",
    "monarch_matmul3", "monarch_matmul3_backward", "monarch_matmulp", "monarch_matmulp_backward",
    "monarch_mixer", "monarch_mixer_workspace_bytes",
    "monarch_mixer_backward", "monarch_mixer_backward_workspace_bytes",
    "monarch_m2_layer", "monarch_m2_layer_workspace_bytes", "monarch_hyena_layer", "monarch_hyena_layer_workspace_bytes",
    "monarch_hyena_heads_layer", "monarch_hyena_heads_layer_workspace_bytes",
    "monarch_blocky_state_bytes", "monarch_blocky_state_offsets", "monarch_blocky_prepare", "monarch_blocky_conv",
    "monarch_fft", "monarch_ifft", "monarch_fft_workspace_bytes",
    "monarch_causal_conv", "monarch_causal_conv_workspace_bytes", "monarch_causal_conv_static",
    "monarch_mlp", "monarch_mlp_workspace_bytes",
]


class MonarchError(RuntimeError):
    def __init__(self, code):
        self.code = code
        msg = _lib.monarch_last_error().decode()
        super().__init__(f"{_lib.monarch_strerror(code).decode()} ({code}): {msg}")


def raw():
    """The ctypes library handle (for tests that exercise the error paths directly)."""
    return _lib


def _check(code):
    if code != OK:
        raise MonarchError(code)


def _dt(t):
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float16:
        return F16
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors must be contiguous device tensors")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _factors(factors):
    arr = (ctypes.c_int * len(factors))(*[int(f) for f in factors])
    return arr, len(factors)


def _workspace(nbytes, ws, device):
    if nbytes == 0:
        return None, 0
    if ws is None:
        ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    if ws.numel() * ws.element_size() < nbytes:
        raise ValueError(f"workspace too small: need {nbytes} bytes")
    return ws, ws.numel() * ws.element_size()


def monarch_permutation_index(b, N):
    out = torch.empty(N, dtype=torch.int32)
    _check(_lib.monarch_permutation_index(b, N, out.data_ptr()))
    return out


def monarch_matmul(x, R, L, out=None):
    nbR, r_out, r_in = R.shape
    nbL, l_out, l_in = L.shape
    batch = x.shape[0]
    y = out if out is not None else torch.empty((batch, nbL * l_out), dtype=x.dtype, device=x.device)
    _check(_lib.monarch_matmul(_ptr(x), _ptr(R), _ptr(L), _ptr(y), batch, nbR, r_out, r_in, nbL, l_out, l_in,
                               _dt(x), None, 0, _stream()))
    return y


def monarch_matmul_backward(x, R, L, dy, need_dx=True, need_dR=True, need_dL=True):
    """(dx, dR, dL) of sum <dy, monarch_matmul(x, R, L)>; dR, dL are float32.  Skipped outputs are None."""
    nbR, r_out, r_in = R.shape
    nbL, l_out, l_in = L.shape
    batch = x.shape[0]
    dx = torch.empty_like(x) if need_dx else None
    dR = torch.empty(R.shape, dtype=torch.float32, device=x.device) if need_dR else None
    dL = torch.empty(L.shape, dtype=torch.float32, device=x.device) if need_dL else None
    _check(_lib.monarch_matmul_backward(_ptr(x), _ptr(R), _ptr(L), _ptr(dy), _ptr(dx), _ptr(dR), _ptr(dL), batch,
                                        nbR, r_out, r_in, nbL, l_out, l_in, _dt(x), None, 0, _stream()))
    return dx, dR, dL


def monarch_matmul3(x, B1, B2, B3, out=None):
    """y = M x for the order-3 Monarch matrix of the factors B1 (first), B2, B3: (b*b, b, b); x: (batch, b^3)."""
    b = B1.shape[-1]
    y = out if out is not None else torch.empty_like(x)
    _check(_lib.monarch_matmul3(_ptr(x), _ptr(B1), _ptr(B2), _ptr(B3), _ptr(y), x.shape[0], b, _dt(x), _stream()))
    return y


def monarch_matmul3_backward(x, B1, B2, B3, dy, need_dx=True, need_dB=True):
    """(dx, dB1, dB2, dB3) of sum <dy, monarch_matmul3(x, B1, B2, B3)>; the factor gradients are float32."""
    b = B1.shape[-1]
    dx = torch.empty_like(x) if need_dx else None
    dB = [torch.empty(B1.shape, dtype=torch.float32, device=x.device) if need_dB else None for _ in range(3)]
    _check(_lib.monarch_matmul3_backward(_ptr(x), _ptr(B1), _ptr(B2), _ptr(B3), _ptr(dy), _ptr(dx), _ptr(dB[0]),
                                         _ptr(dB[1]), _ptr(dB[2]), x.shape[0], b, _dt(x), _stream()))
    return (dx, *dB)


def monarch_matmulp(x, B, out=None):
    """y = M x for the order-p Monarch matrix of the factors B: (p, b^(p-1), b, b), B[0] applied first; x: (batch, b^p)."""
    p, b = B.shape[0], B.shape[-1]
    y = out if out is not None else torch.empty_like(x)
    _check(_lib.monarch_matmulp(_ptr(x), _ptr(B), _ptr(y), x.shape[0], b, p, _dt(x), _stream()))
    return y


def monarch_matmulp_backward(x, B, dy, need_dx=True, need_dB=True):
    """(dx, dB) of sum <dy, monarch_matmulp(x, B)>; dB is float32."""
    p, b = B.shape[0], B.shape[-1]
    dx = torch.empty_like(x) if need_dx else None
    dB = torch.empty(B.shape, dtype=torch.float32, device=x.device) if need_dB else None
    _check(_lib.monarch_matmulp_backward(_ptr(x), _ptr(B), _ptr(dy), _ptr(dx), _ptr(dB), x.shape[0], b, p, _dt(x), _stream()))
    return dx, dB


def monarch_mixer(u, K, g_in, g_out, R1, L1, R2, L2, out=None):
    """y = g_out * M2(K[h] * M1(g_in * u)) with M = P L P R P square; u, gates, y: (B, H, N); K: (H, N)."""
    B, H, N = u.shape
    bs = R1.shape[0]
    y = out if out is not None else torch.empty_like(u)
    _check(_lib.monarch_mixer(_ptr(u), _ptr(K), _ptr(g_in), _ptr(g_out), _ptr(R1), _ptr(L1), _ptr(R2), _ptr(L2), _ptr(y),
                              B, H, bs, _dt(u), None, 0, _stream()))
    return y


def monarch_mixer_backward(u, K, g_in, g_out, R1, L1, R2, L2, dy, ws=None):
    """Gradients of sum <dy, monarch_mixer(...)>: dict with du, dK, dg_in, dg_out (None without the gate), dR1, dL1,
    dR2, dL2; dK and the factor gradients are float32."""
    B, H, N = u.shape
    bs = R1.shape[0]
    f32 = dict(dtype=torch.float32, device=u.device)
    g = {"du": torch.empty_like(u), "dK": torch.empty((H, N), **f32),
         "dg_in": torch.empty_like(u) if g_in is not None else None,
         "dg_out": torch.empty_like(u) if g_out is not None else None}
    for name in ("dR1", "dL1", "dR2", "dL2"):
        g[name] = torch.empty((bs, bs, bs), **f32)
    ws, wsb = _workspace(_lib.monarch_mixer_backward_workspace_bytes(B, H, bs, _dt(u)), ws, u.device)
    _check(_lib.monarch_mixer_backward(_ptr(u), _ptr(K), _ptr(g_in), _ptr(g_out), _ptr(R1), _ptr(L1), _ptr(R2), _ptr(L2),
                                       _ptr(dy), _ptr(g["du"]), _ptr(g["dK"]), _ptr(g["dg_in"]), _ptr(g["dg_out"]),
                                       _ptr(g["dR1"]), _ptr(g["dL1"]), _ptr(g["dR2"]), _ptr(g["dL2"]), B, H, bs, _dt(u),
                                       _ptr(ws), wsb, _stream()))
    return g


def monarch_m2_layer_workspace_bytes(B, n, d, dt=F32):
    return _lib.monarch_m2_layer_workspace_bytes(B, n, d, dt)


def monarch_m2_layer(x, seq, n_kernel, dim, d_kernel, gamma, beta, eps=1e-5, act=1, ws=None, out=None):
    """LayerNorm(M4 act(k_d * M3 X~) + X~), X~ = (M2 act(K_n * M1 x^T))^T; x: (B, n, d); seq = (R1, L1, R2, L2),
    dim = (R3, L3, R4, L4)."""
    B, n, d = x.shape
    bn, bd = seq[0].shape[0], dim[0].shape[0]
    y = out if out is not None else torch.empty_like(x)
    need = _lib.monarch_m2_layer_workspace_bytes(B, n, d, _dt(x))
    ws, wsb = _workspace(max(need, 16), ws, x.device)
    _check(_lib.monarch_m2_layer(_ptr(x), _ptr(y), B, bn, bd, *(_ptr(t) for t in seq), _ptr(n_kernel),
                                 *(_ptr(t) for t in dim), _ptr(d_kernel), _ptr(gamma), _ptr(beta), eps, act, _dt(x),
                                 _ptr(ws), wsb, _stream()))
    return y


def monarch_hyena_layer_workspace_bytes(B, n, d, klen, factors, torch_dtype):
    f, nf = _factors(factors)
    nfft = 1
    for v in factors:
        nfft *= int(v)
    dt = {torch.float32: F32, torch.bfloat16: BF16}[torch_dtype]
    return _lib.monarch_hyena_layer_workspace_bytes(B, n, d, klen, nfft, f, nf, dt)


def monarch_hyena_layer(u, W_in, b_in, k_short, k_long, W_out, b_out, factors, causal=True, ws=None, out=None):
    """W_out (X1~ * conv(k_long, X2~ * V~)) + b_out with [X1; X2; V] = W_in u + b_in passed through short causal
    depthwise convolutions; u: (B, n, d)."""
    B, n, d = u.shape
    f, nf = _factors(factors)
    nfft = 1
    for v in factors:
        nfft *= int(v)
    taps, klen = k_short.shape[1], k_long.shape[1]
    y = out if out is not None else torch.empty_like(u)
    need = _lib.monarch_hyena_layer_workspace_bytes(B, n, d, klen, nfft, f, nf, _dt(u))
    ws, wsb = _workspace(max(need, 16), ws, u.device)
    _check(_lib.monarch_hyena_layer(_ptr(u), _ptr(W_in), _ptr(b_in), _ptr(k_short), _ptr(k_long), _ptr(W_out), _ptr(b_out),
                                    _ptr(y), B, n, d, taps, klen, nfft, f, nf, 1 if causal else 0, _dt(u), _ptr(ws), wsb,
                                    _stream()))
    return y


def monarch_hyena_heads_layer_workspace_bytes(B, n, d, klen, factors, head_dim, torch_dtype):
    f, nf = _factors(factors)
    nfft = 1
    for v in factors:
        nfft *= int(v)
    dt = {torch.float32: F32, torch.bfloat16: BF16}[torch_dtype]
    return _lib.monarch_hyena_heads_layer_workspace_bytes(B, n, d, klen, nfft, f, nf, head_dim, dt)


def monarch_hyena_heads_layer(u, W_in, b_in, k_short, k_long, W_out, b_out, factors, head_dim, causal=True, ws=None, out=None):
    """monarch_hyena_layer with heads of head_dim features: k_long (d / head_dim, klen), per head
    O[j] = sum_i X1~[i] * conv(k_long[head], X2~[i] * V~[j]); u: (B, n, d)."""
    B, n, d = u.shape
    f, nf = _factors(factors)
    nfft = 1
    for v in factors:
        nfft *= int(v)
    taps, klen = k_short.shape[1], k_long.shape[1]
    y = out if out is not None else torch.empty_like(u)
    need = _lib.monarch_hyena_heads_layer_workspace_bytes(B, n, d, klen, nfft, f, nf, head_dim, _dt(u))
    ws, wsb = _workspace(max(need, 16), ws, u.device)
    _check(_lib.monarch_hyena_heads_layer(_ptr(u), _ptr(W_in), _ptr(b_in), _ptr(k_short), _ptr(k_long), _ptr(W_out), _ptr(b_out),
                                          _ptr(y), B, n, d, taps, klen, nfft, f, nf, 1 if causal else 0, head_dim, _dt(u),
                                          _ptr(ws), wsb, _stream()))
    return y


def monarch_blocky_prepare(Lt, Rt, k, mask=True, state=None):
    """State (uint8 device tensor) of the polynomial-parameterised Monarch convolution: Lt, Rt (N, bs), k (H, klen),
    all float32."""
    N, bs = Lt.shape
    H, klen = k.shape
    need = _lib.monarch_blocky_state_bytes(H, bs)
    if state is None:
        state = torch.empty(max(need, 16), dtype=torch.uint8, device=Lt.device)
    _check(_lib.monarch_blocky_prepare(_ptr(Lt), _ptr(Rt), _ptr(k), H, klen, bs, int(bool(mask)), _ptr(state),
                                       state.numel(), _stream()))
    return state


def monarch_blocky_conv(u, g_in, g_out, state, bs, out=None):
    B, H, n = u.shape
    y = out if out is not None else torch.empty_like(u)
    _check(_lib.monarch_blocky_conv(_ptr(u), _ptr(g_in), _ptr(g_out), _ptr(state), state.numel(), _ptr(y), B, H, n, bs,
                                    _dt(u), _stream()))
    return y


def blocky_state_views(state, H, bs):
    """The parts of a prepared state as complex64 tensors (R1, L1, R2, L2: (bs, bs, bs); Kf: (H, N)), for tests."""
    N = bs * bs
    off = (ctypes.c_size_t * 5)()
    _check(_lib.monarch_blocky_state_offsets(H, bs, off))
    parts = [state[off[i]:off[i] + N * bs * 8].view(torch.complex64).reshape(bs, bs, bs) for i in range(4)]
    parts.append(state[off[4]:off[4] + H * N * 8].view(torch.complex64).reshape(H, N))
    return parts


def monarch_fft_workspace_bytes(rows, N, factors, dt=F32):
    f, nf = _factors(factors)
    return _lib.monarch_fft_workspace_bytes(rows, N, f, nf, dt)


def monarch_fft(x, factors, real_input, ws=None, out=None):
    f, nf = _factors(factors)
    N = 1
    for v in factors:
        N *= int(v)
    rows = x.numel() // (N if real_input else 2 * N)
    X = out if out is not None else torch.empty((rows, N, 2), dtype=torch.float32, device=x.device)
    ws, nbytes = _workspace(_lib.monarch_fft_workspace_bytes(rows, N, f, nf, _dt(x)), ws, x.device)
    _check(_lib.monarch_fft(_ptr(x), _ptr(X), rows, N, f, nf, 1 if real_input else 0, _dt(x),
                            _ptr(ws), nbytes, _stream()))
    return X


def monarch_ifft(X, factors, real_output, dtype=torch.float32, ws=None, out=None):
    f, nf = _factors(factors)
    N = 1
    for v in factors:
        N *= int(v)
    rows = X.numel() // (2 * N)
    shape = (rows, N) if real_output else (rows, N, 2)
    x = out if out is not None else torch.empty(shape, dtype=dtype, device=X.device)
    ws, nbytes = _workspace(_lib.monarch_fft_workspace_bytes(rows, N, f, nf, _dt(x)), ws, X.device)
    _check(_lib.monarch_ifft(_ptr(X), _ptr(x), rows, N, f, nf, 1 if real_output else 0, _dt(x),
                             _ptr(ws), nbytes, _stream()))
    return x


def monarch_causal_conv_workspace_bytes(B, H, n, klen, factors, dt):
    f, nf = _factors(factors)
    nfft = 1
    for v in factors:
        nfft *= int(v)
    return _lib.monarch_causal_conv_workspace_bytes(B, H, n, klen, nfft, f, nf, dt)


def monarch_causal_conv(u, k, g_in, g_out, factors, causal=True, ws=None, out=None):
    B, H, n = u.shape
    klen = k.shape[1]
    f, nf = _factors(factors)
    nfft = 1
    for v in factors:
        nfft *= int(v)
    y = out if out is not None else torch.empty_like(u)
    ws, nbytes = _workspace(_lib.monarch_causal_conv_workspace_bytes(B, H, n, klen, nfft, f, nf, _dt(u)), ws, u.device)
    _check(_lib.monarch_causal_conv(_ptr(u), _ptr(k), _ptr(g_in), _ptr(g_out), _ptr(y), B, H, n, klen, nfft,
                                    f, nf, 1 if causal else 0, _dt(u), _ptr(ws), nbytes, _stream()))
    return y


STATIC_SCRATCH_BYTES = 32 << 20   # MONARCH_STATIC_SCRATCH_BYTES of the header


def monarch_causal_conv_static(u, k, g_in, g_out, factors, out, causal=True):
    """The entry point that allocates nothing: the caller passes the output too; scratch is the library's own."""
    B, H, n = u.shape
    f, nf = _factors(factors)
    nfft = 1
    for v in factors:
        nfft *= int(v)
    _check(_lib.monarch_causal_conv_static(_ptr(u), _ptr(k), _ptr(g_in), _ptr(g_out), _ptr(out), B, H, n, k.shape[1], nfft,
                                           f, nf, 1 if causal else 0, _dt(u), _stream()))
    return out


def monarch_mlp_workspace_bytes(tokens, d, d_hidden, nb, order, mid1=0, mid2=0, dt=BF16):
    return _lib.monarch_mlp_workspace_bytes(tokens, d, d_hidden, nb, order, mid1, mid2, dt)


def monarch_mlp(x, W1_R, W1_L, b1, W2_R, W2_L, b2, nb, order, act, d_hidden, mid1=0, mid2=0, ws=None, out=None):
    tokens, d = x.shape
    y = out if out is not None else torch.empty_like(x)
    ws, nbytes = _workspace(_lib.monarch_mlp_workspace_bytes(tokens, d, d_hidden, nb, order, mid1, mid2, _dt(x)),
                            ws, x.device)
    _check(_lib.monarch_mlp(_ptr(x), _ptr(y), tokens, d, d_hidden, nb, order, _ptr(W1_R), _ptr(W1_L), _ptr(b1),
                            _ptr(W2_R), _ptr(W2_L), _ptr(b2), mid1, mid2, act, _dt(x), _ptr(ws), nbytes, _stream()))
    return y
