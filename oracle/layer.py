"""CPU oracle for the basic M2 layer (Sec. 3.2, Eq. 2 and its dimension-mixing counterpart, with the
non-linearity, skip connection and layer normalisation of the paper's basic implementation).

TEST INFRASTRUCTURE ONLY.  Plain numpy float64 with the four Monarch matrices materialised densely
(oracle.monarch_dense), so that every step is a dense matrix product or an elementwise operation:
    X~ = ( M2 act( K_n o (M1 X^T) ) )^T           mix along the sequence, one kernel row per feature
    Y  = M4 act( k_d o (M3 X~) )                  mix along the features, one kernel shared by all positions
    out = LayerNorm(Y + X~)                       over the features, biased variance, affine
X: (B, n, d); M1, M2: n x n; M3, M4: d x d; K_n: (d, n); k_d: (d,).  Factor roles as in monarch_matmul: R is the
factor applied first.
"""
import numpy as np

from . import monarch_dense


def _act(a, act):
    if act == "relu":
        return np.maximum(a, 0.0)
    assert act == "none"
    return a


def m2_layer(x, seq, n_kernel, dim, d_kernel, gamma, beta, eps=1e-5, act="relu"):
    """seq = (R1, L1, R2, L2), dim = (R3, L3, R4, L4).  Returns (out, X~)."""
    x = np.asarray(x, dtype=np.float64)
    M1, M2 = monarch_dense(seq[0], seq[1]), monarch_dense(seq[2], seq[3])
    M3, M4 = monarch_dense(dim[0], dim[1]), monarch_dense(dim[2], dim[3])
    Kn, kd = np.asarray(n_kernel, dtype=np.float64), np.asarray(d_kernel, dtype=np.float64)
    xt = x.transpose(0, 2, 1)                                           # (B, d, n)
    s = _act(np.einsum("ij,bhj->bhi", M1, xt) * Kn[None], act)
    xtil = np.einsum("ij,bhj->bhi", M2, s).transpose(0, 2, 1)           # (B, n, d)
    z = _act(np.einsum("ij,btj->bti", M3, xtil) * kd[None, None], act)
    r = np.einsum("ij,btj->bti", M4, z) + xtil
    mean = r.mean(axis=-1, keepdims=True)
    var = ((r - mean) ** 2).mean(axis=-1, keepdims=True)
    out = (r - mean) / np.sqrt(var + eps) * np.asarray(gamma, dtype=np.float64) + np.asarray(beta, dtype=np.float64)
    return out, xtil


def mixer_backward(u, K, g_in, g_out, R1, L1, R2, L2, dy):
    """Gradients of S = sum <dy, y>, y = g_out o M2 (K[h] o M1 (g_in o u)) (the sequence mixer of Sec. 3.2 Eq. 2 in
    its gated form), by the chain rule through its five steps with the dense Monarch matrices; the gradients of the
    block-diagonal factors come from the order-2 product's own oracle (oracle.matmul_backward).
    Returns a dict: du, dK, dg_in, dg_out (None without the gate), dR1, dL1, dR2, dL2."""
    from . import matmul_backward
    u, K, dy = (np.asarray(t, dtype=np.float64) for t in (u, K, dy))
    B, H, N = u.shape
    gi = np.asarray(g_in, dtype=np.float64) if g_in is not None else None
    go = np.asarray(g_out, dtype=np.float64) if g_out is not None else None
    M1, M2 = monarch_dense(R1, L1), monarch_dense(R2, L2)
    a = u * gi if gi is not None else u
    s = a @ M1.T
    t = s * K[None]
    w = t @ M2.T
    dw = dy * go if go is not None else dy
    out = {"dg_out": dy * w if go is not None else None}
    dt = dw @ M2
    _, out["dR2"], out["dL2"] = matmul_backward(t.reshape(B * H, N), R2, L2, dw.reshape(B * H, N))
    out["dK"] = (dt * s).sum(axis=0)
    ds = dt * K[None]
    da = ds @ M1
    _, out["dR1"], out["dL1"] = matmul_backward(a.reshape(B * H, N), R1, L1, ds.reshape(B * H, N))
    out["du"] = da * gi if gi is not None else da
    out["dg_in"] = da * u if gi is not None else None
    return out


def hyena_layer(u, W_in, b_in, k_short, k_long, W_out, b_out, nfft=None, causal=True):
    """The paper's gated-convolution layer (appendix algorithm "M2 Hyena layer with heads" at head dimension 1; with
    causal=False the bidirectional gated convolution of the M2-BERT sequence mixer), step by step in float64:
        [X1; X2; V] = W_in u_t + b_in                 three projections of every position (W_in: (3d, d))
        X1~, X2~, V~ = short causal depthwise convolutions along the sequence (k_short: (3d, ks)):
                       x~[c, t] = sum_tau k_short[c, tau] x[c, t - tau]
        O = X1~ o conv(k_long, X2~ o V~)              the gated long convolution, one kernel row per feature
        y_t = W_out O[:, t] + b_out
    u: (B, n, d); returns (B, n, d).  The long convolution is oracle.causal_conv (the direct sum)."""
    from . import causal_conv
    u = np.asarray(u, dtype=np.float64)
    B, n, d = u.shape
    W_in, W_out = np.asarray(W_in, dtype=np.float64), np.asarray(W_out, dtype=np.float64)
    proj = np.einsum("cj,btj->bct", W_in, u)                           # (B, 3d, n)
    if b_in is not None:
        proj = proj + np.asarray(b_in, dtype=np.float64)[None, :, None]
    ks = np.asarray(k_short, dtype=np.float64)
    short = np.zeros_like(proj)
    for tau in range(ks.shape[1]):                                     # x~[c, t] += k[c, tau] x[c, t - tau]
        short[:, :, tau:] += ks[None, :, tau, None] * proj[:, :, :n - tau]
    x1, x2, v = short[:, :d], short[:, d:2 * d], short[:, 2 * d:]
    o = causal_conv(v, k_long, x2, x1, nfft=nfft, causal=causal)       # (B, d, n)
    y = np.einsum("cj,bjt->btc", W_out, o)
    if b_out is not None:
        y = y + np.asarray(b_out, dtype=np.float64)[None, None, :]
    return y


def hyena_heads_layer(u, W_in, b_in, k_short, k_long, W_out, b_out, head_dim, nfft=None, causal=True):
    """The same layer with heads (appendix algorithm "M2 Hyena layer with heads"), step by step in float64: the d
    features are d / head_dim heads of head_dim consecutive features, k_long has one row per head, and for every head
        XV[i][j] = conv(k_long[head], X2~[i] o V~[j])     outer product per position, convolved along the sequence
        O[j]     = sum_i X1~[i] o XV[i][j]                 the row vector X1~ times the matrix XV, per position
    with i, j < head_dim numbering the head's features; projections, short convolutions and the output projection as in
    hyena_layer.  u: (B, n, d); returns (B, n, d)."""
    from . import causal_conv
    u = np.asarray(u, dtype=np.float64)
    B, n, d = u.shape
    dh = int(head_dim)
    assert d % dh == 0
    heads = d // dh
    W_in, W_out = np.asarray(W_in, dtype=np.float64), np.asarray(W_out, dtype=np.float64)
    proj = np.einsum("cj,btj->bct", W_in, u)
    if b_in is not None:
        proj = proj + np.asarray(b_in, dtype=np.float64)[None, :, None]
    ks = np.asarray(k_short, dtype=np.float64)
    short = np.zeros_like(proj)
    for tau in range(ks.shape[1]):
        short[:, :, tau:] += ks[None, :, tau, None] * proj[:, :, :n - tau]
    x1, x2, v = (short[:, m * d:(m + 1) * d].reshape(B, heads, dh, n) for m in range(3))
    o = np.zeros((B, heads, dh, n))
    for i in range(dh):
        for j in range(dh):
            xv = causal_conv(x2[:, :, i] * v[:, :, j], k_long, None, None, nfft=nfft, causal=causal)   # (B, heads, n)
            o[:, :, j] += x1[:, :, i] * xv
    y = np.einsum("cj,bjt->btc", W_out, o.reshape(B, d, n))
    if b_out is not None:
        y = y + np.asarray(b_out, dtype=np.float64)[None, None, :]
    return y
