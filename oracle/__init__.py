"""ctypes front end of the CPU oracle (oracle/monarch_oracle.c).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the cpu_baseline leg of
the benchmark call this; the product path never does.  The wrappers only
marshal numpy arrays (float64 / complex128, C-contiguous) into the C
functions; all arithmetic lives in the C file.  (oracle/blocky.py, plain numpy, holds the
polynomial-parameterised Monarch matrices and their convolution.)
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "monarch_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force=False):
    """Compile the oracle with gcc (plain C99, -O2, OpenMP over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-std=c99", "-Wall", "-Wextra", "-shared", "-fPIC",
             _SRC, "-o", _LIB, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _c128(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.complex128))


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def num_threads():
    return int(lib().oracle_num_threads())


def perm(b, N):
    """sigma_(b,N) as an int32 vector: (P_(b,N) x)[i] = x[sigma[i]]."""
    out = np.empty(N, dtype=np.int32)
    rc = lib().oracle_perm(ctypes.c_int(b), ctypes.c_int(N), _p(out))
    if rc != 0:
        raise ValueError("b must divide N")
    return out


def monarch_dense(R, L):
    """Dense d_out x d_in matrix of P3 L P2 R P1; R, L are [block][out][in]."""
    cplx = np.iscomplexobj(R) or np.iscomplexobj(L)
    R = _c128(R) if cplx else _f64(R)
    L = _c128(L) if cplx else _f64(L)
    nbR, r_out, r_in = R.shape
    nbL, l_out, l_in = L.shape
    M = np.empty((nbL * l_out, nbR * r_in), dtype=R.dtype)
    fn = lib().oracle_monarch_dense_c if cplx else lib().oracle_monarch_dense
    rc = fn(_p(R), _p(L), ctypes.c_int(nbR), ctypes.c_int(r_out), ctypes.c_int(r_in),
            ctypes.c_int(nbL), ctypes.c_int(l_out), ctypes.c_int(l_in), _p(M))
    if rc != 0:
        raise ValueError("inconsistent Monarch factor shapes")
    return M


def matmul(x, R, L):
    """y[v] = (P3 L P2 R P1) x[v] with the matrix materialised densely."""
    x, R, L = _f64(x), _f64(R), _f64(L)
    nbR, r_out, r_in = R.shape
    nbL, l_out, l_in = L.shape
    batch = x.shape[0]
    assert x.shape[1] == nbR * r_in
    y = np.empty((batch, nbL * l_out), dtype=np.float64)
    rc = lib().oracle_matmul(_p(x), _p(R), _p(L), _p(y), ctypes.c_int64(batch),
                             ctypes.c_int(nbR), ctypes.c_int(r_out), ctypes.c_int(r_in),
                             ctypes.c_int(nbL), ctypes.c_int(l_out), ctypes.c_int(l_in))
    if rc != 0:
        raise ValueError("inconsistent Monarch factor shapes")
    return y


def matmul_backward(x, R, L, dy):
    """(dx, dR, dL) of S = sum_v <dy[v], M x[v]>, M = P3 L P2 R P1, by the chain rule through the five steps."""
    x, R, L, dy = _f64(x), _f64(R), _f64(L), _f64(dy)
    nbR, r_out, r_in = R.shape
    nbL, l_out, l_in = L.shape
    batch = x.shape[0]
    assert x.shape[1] == nbR * r_in and dy.shape == (batch, nbL * l_out)
    dx, dR, dL = np.empty_like(x), np.empty_like(R), np.empty_like(L)
    rc = lib().oracle_matmul_backward(_p(x), _p(R), _p(L), _p(dy), _p(dx), _p(dR), _p(dL), ctypes.c_int64(batch),
                                      ctypes.c_int(nbR), ctypes.c_int(r_out), ctypes.c_int(r_in),
                                      ctypes.c_int(nbL), ctypes.c_int(l_out), ctypes.c_int(l_in))
    if rc != 0:
        raise ValueError("inconsistent Monarch factor shapes")
    return dx, dR, dL


def mixer(u, K, g_in, g_out, R1, L1, R2, L2):
    """y = g_out o M2 (K[h] o M1 (g_in o u)) with two general square order-2 Monarch matrices (Sec. 3.2 Eq. 2).
    u, gates: (B, H, N); K: (H, N); factors (b, b, b), N = b*b."""
    u, K = _f64(u), _f64(K)
    B, H, N = u.shape
    b = R1.shape[0]
    assert N == b * b and K.shape == (H, N)
    R1, L1, R2, L2 = _f64(R1), _f64(L1), _f64(R2), _f64(L2)
    gi = _f64(g_in) if g_in is not None else None
    go = _f64(g_out) if g_out is not None else None
    y = np.empty_like(u)
    rc = lib().oracle_mixer(_p(u), _p(K), _p(gi) if gi is not None else None, _p(go) if go is not None else None,
                            _p(R1), _p(L1), _p(R2), _p(L2), _p(y), ctypes.c_int64(B * H), ctypes.c_int(H), ctypes.c_int(b))
    if rc != 0:
        raise ValueError("inconsistent mixer shapes")
    return y


def dft(x):
    """X[r,m] = sum_j x[r,j] omega_N^(m j), omega_N = exp(+2 pi i / N); O(N^2) per row."""
    x = _c128(x)
    x2 = x.reshape(-1, x.shape[-1])
    X = np.empty_like(x2)
    lib().oracle_dft(_p(x2), _p(X), ctypes.c_int64(x2.shape[0]), ctypes.c_int(x2.shape[1]))
    return X.reshape(x.shape)


def dft_bins(x, bins):
    """Selected output bins of dft(x): X[r, bins[q]] for every row (for sizes where O(N^2) is too slow)."""
    x = _c128(x)
    x2 = x.reshape(-1, x.shape[-1])
    bins = np.ascontiguousarray(np.asarray(bins, dtype=np.int32))
    out = np.empty((x2.shape[0], bins.shape[0]), dtype=np.complex128)
    lib().oracle_dft_bins(_p(x2), _p(out), ctypes.c_int64(x2.shape[0]), ctypes.c_int(x2.shape[1]),
                          _p(bins), ctypes.c_int(bins.shape[0]))
    return out


def idft(X):
    """Inverse of dft: x[r,j] = (1/N) sum_m X[r,m] omega_N^(-m j)."""
    X = _c128(X)
    X2 = X.reshape(-1, X.shape[-1])
    x = np.empty_like(X2)
    lib().oracle_idft(_p(X2), _p(x), ctypes.c_int64(X2.shape[0]), ctypes.c_int(X2.shape[1]))
    return x.reshape(X.shape)


def dft_factors(N1, N2):
    """(R, L) complex block-diagonal factors whose order-2 Monarch product is F_(N1*N2)."""
    N = N1 * N2
    R = np.empty((N2, N1, N1), dtype=np.complex128)
    L = np.empty((N1, N2, N2), dtype=np.complex128)
    lib().oracle_dft_factors(ctypes.c_int(N1), ctypes.c_int(N2), _p(R), _p(L))
    assert R.size == N * N1 and L.size == N * N2
    return R, L


def monarch_dft_dense(N1, N2):
    N = N1 * N2
    M = np.empty((N, N), dtype=np.complex128)
    rc = lib().oracle_monarch_dft_dense(ctypes.c_int(N1), ctypes.c_int(N2), _p(M))
    assert rc == 0
    return M


def monarch3_dense(B1, B2, B3):
    """Dense matrix of the order-3 product P^R B3 P B2 P B1 P^R, N = b^3."""
    B1, B2, B3 = _c128(B1), _c128(B2), _c128(B3)
    b = B1.shape[-1]
    assert B1.shape == B2.shape == B3.shape == (b * b, b, b)
    N = b ** 3
    M = np.empty((N, N), dtype=np.complex128)
    rc = lib().oracle_monarch3_dense_c(_p(B1), _p(B2), _p(B3), ctypes.c_int(b), _p(M))
    assert rc == 0
    return M


def dft3_factors(b):
    shape = (b * b, b, b)
    B1 = np.empty(shape, dtype=np.complex128)
    B2 = np.empty(shape, dtype=np.complex128)
    B3 = np.empty(shape, dtype=np.complex128)
    lib().oracle_dft3_factors(ctypes.c_int(b), _p(B1), _p(B2), _p(B3))
    return B1, B2, B3


def monarch3_dft_dense(b):
    N = b ** 3
    M = np.empty((N, N), dtype=np.complex128)
    rc = lib().oracle_monarch3_dft_dense(ctypes.c_int(b), _p(M))
    assert rc == 0
    return M


def causal_conv(u, k, g_in=None, g_out=None, nfft=None, causal=True):
    """Direct-sum long convolution with optional gates; u: (B,H,n), k: (H,klen)."""
    u, k = _f64(u), _f64(k)
    B, H, n = u.shape
    assert k.shape[0] == H
    klen = k.shape[1]
    if nfft is None:
        nfft = 2 * n
    g_in = None if g_in is None else _f64(g_in)
    g_out = None if g_out is None else _f64(g_out)
    y = np.empty_like(u)
    lib().oracle_causal_conv(_p(u), _p(k), _p(g_in), _p(g_out), _p(y), ctypes.c_int(B),
                             ctypes.c_int(H), ctypes.c_int(n), ctypes.c_int(klen),
                             ctypes.c_int(nfft), ctypes.c_int(1 if causal else 0))
    return y


def causal_conv_points(u, k, g_in, g_out, rows, ts, nfft=None, causal=True):
    """Single outputs y[b, h, t] of causal_conv: rows[i] = b * H + h, ts[i] = t (for rows too long to sum whole)."""
    u, k = _f64(u), _f64(k)
    B, H, n = u.shape
    klen = k.shape[1]
    if nfft is None:
        nfft = 2 * n
    g_in = None if g_in is None else _f64(g_in)
    g_out = None if g_out is None else _f64(g_out)
    rows = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
    ts = np.ascontiguousarray(np.asarray(ts, dtype=np.int32))
    assert rows.shape == ts.shape and rows.ndim == 1
    assert rows.min(initial=0) >= 0 and rows.max(initial=0) < B * H and ts.min(initial=0) >= 0 and ts.max(initial=0) < n
    out = np.empty(rows.shape[0], dtype=np.float64)
    lib().oracle_causal_conv_points(_p(u), _p(k), _p(g_in), _p(g_out), _p(out), ctypes.c_int(B), ctypes.c_int(H),
                                    ctypes.c_int(n), ctypes.c_int(klen), ctypes.c_int(nfft),
                                    ctypes.c_int(1 if causal else 0), _p(rows), _p(ts), ctypes.c_int(rows.shape[0]))
    return out


def fft_conv_row(u, k, nfft):
    """(F^-1((F k') o (F u'))) over all nfft outputs for one row, via the naive DFT."""
    u, k = _f64(u), _f64(k)
    y = np.empty(nfft, dtype=np.complex128)
    lib().oracle_fft_conv_row(_p(u), _p(k), _p(y), ctypes.c_int(u.shape[0]),
                              ctypes.c_int(k.shape[0]), ctypes.c_int(nfft))
    return y


def mlp(x, W1_R, W1_L, b1, W2_R, W2_L, b2, nb, order, act, mid1=0, mid2=0):
    """y = W2 act(W1 x + b1) + b2 with W1, W2 dense-materialised; x: (tokens, d)."""
    x = _f64(x)
    tokens, d = x.shape
    W1_R, W2_R = _f64(W1_R), _f64(W2_R)
    W1_L = None if W1_L is None else _f64(W1_L)
    W2_L = None if W2_L is None else _f64(W2_L)
    b1 = None if b1 is None else _f64(b1)
    b2 = None if b2 is None else _f64(b2)
    if order == 1:
        d_hidden = W1_R.shape[0] * W1_R.shape[1]
    else:
        d_hidden = W1_L.shape[0] * W1_L.shape[1]
        mid1 = mid1 or W1_R.shape[0] * W1_R.shape[1]
        mid2 = mid2 or W2_R.shape[0] * W2_R.shape[1]
    y = np.empty((tokens, d), dtype=np.float64)
    rc = lib().oracle_mlp(_p(x), _p(y), ctypes.c_int64(tokens), ctypes.c_int(d),
                          ctypes.c_int(d_hidden), ctypes.c_int(nb), ctypes.c_int(order),
                          _p(W1_R), _p(W1_L), _p(b1), _p(W2_R), _p(W2_L), _p(b2),
                          ctypes.c_int(mid1), ctypes.c_int(mid2), ctypes.c_int(act))
    if rc != 0:
        raise ValueError("inconsistent MLP shapes")
    return y
