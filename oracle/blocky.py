"""CPU oracle for the polynomial-parameterised ("blocky") Monarch matrices and the convolution built on
them (appendix: the blocky-Monarch algorithm, the causal coefficient masks, the blocky Monarch convolution).

TEST INFRASTRUCTURE ONLY, like the rest of this package.  Plain numpy in float64 / complex128: the
definitions written out, dense matrices, a library solve for the inverse.  Notation: b = sqrt(N),
omega_m = exp(+2 pi i / m), an index i = i1 b + i0.
"""
import numpy as np

from . import perm


def blocky_monarch(Lt, Rt):
    """(L, R): the block-diagonal factors that the coefficient matrices Lt, Rt (N x b, real) stand for, as
    complex arrays [block][row][column]  (equations for the blocks of R and of L in the blocky section):
      R_{j1}[i0, j0] = r~_{j1,j0}(omega_b^{i0}),            r~_{j1,j0}(Y) = sum_{a<b} Rt[j1 b + a, j0] Y^a
      L_{i0}[i1, j1] = l_{j1}(omega_N^{i1 b + i0}),          l_{j1}(Z)    = sum_{a<N} Lt[a, j1] Z^a
    (the evaluation point of L follows the blocky-Monarch algorithm, L' = P F_N Lt: row i0 b + i1 of L' is
    row i1 b + i0 of F_N Lt)."""
    Lt, Rt = np.asarray(Lt, dtype=np.float64), np.asarray(Rt, dtype=np.float64)
    N, b = Lt.shape
    assert b * b == N and Rt.shape == (N, b)
    R = np.empty((b, b, b), dtype=np.complex128)
    L = np.empty((b, b, b), dtype=np.complex128)
    a_b, a_N = np.arange(b), np.arange(N)
    for j1 in range(b):
        for i0 in range(b):
            point = np.exp(2j * np.pi * ((i0 * a_b) % b) / b)          # omega_b^(i0 a)
            R[j1, i0, :] = point @ Rt[j1 * b:(j1 + 1) * b, :]
    for i0 in range(b):
        for i1 in range(b):
            point = np.exp(2j * np.pi * (((i1 * b + i0) * a_N) % N) / N)   # omega_N^((i1 b + i0) a)
            L[i0, i1, :] = point @ Lt
    return L, R


def causal_mask(Lt, Rt):
    """The masked coefficient matrices of the degree lemma: of Lt only the top b x b block survives, and of it
    the entries [a, j1] with a >= j1; of every block of Rt the entries [a, j0] with a >= j0, except those with
    a >= floor(b/2) in a column j0 < floor(b/2)."""
    Lt, Rt = np.array(Lt, dtype=np.float64), np.array(Rt, dtype=np.float64)
    N, b = Lt.shape
    half = b // 2
    Lm = np.zeros_like(Lt)
    for a in range(b):
        for j1 in range(b):
            if a >= j1:
                Lm[a, j1] = Lt[a, j1]
    Rm = np.zeros_like(Rt)
    for j1 in range(b):
        for a in range(b):
            for j0 in range(b):
                if a < j0 or (a >= half and j0 < half):
                    continue
                Rm[j1 * b + a, j0] = Rt[j1 * b + a, j0]
    return Lm, Rm


def dense_from_blocks(L, R):
    """M = P L P R P (Sec. 3.1) with the dense permutation and the dense block-diagonal matrices, complex."""
    b = L.shape[0]
    N = b * b
    P = np.zeros((N, N))
    P[np.arange(N), perm(b, N)] = 1.0
    Ld = np.zeros((N, N), dtype=np.complex128)
    Rd = np.zeros((N, N), dtype=np.complex128)
    for k in range(b):
        Ld[k * b:(k + 1) * b, k * b:(k + 1) * b] = L[k]
        Rd[k * b:(k + 1) * b, k * b:(k + 1) * b] = R[k]
    return P @ Ld @ P @ Rd @ P


def inverse_blocks(L, R):
    """Factors of M^-1 = P R^-1 P L^-1 P in the roles of monarch_matmul: (L2, R2) = (blockwise R^-1, blockwise
    L^-1); R2 is applied first."""
    return np.stack([np.linalg.inv(x) for x in R]), np.stack([np.linalg.inv(x) for x in L])


def blocky_monarch_conv(Lt, Rt, k, u, g_in=None, g_out=None, mask=True):
    """The blocky Monarch convolution with gates, per row of u (B, H, n) and channel kernel k (H, klen):
      L, R = blocky_monarch(masked Lt, Rt);  M = P L P R P
      f = M^-1 ( (M (k, 0)) o (M (g_in o u, 0)) );  y = g_out o Re f[0:n]
    n, klen <= N.  (f is real up to rounding: it holds the coefficients of a real polynomial in a real basis.)"""
    if mask:
        Lt, Rt = causal_mask(Lt, Rt)
    L, R = blocky_monarch(Lt, Rt)
    M = dense_from_blocks(L, R)
    u = np.asarray(u, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    B, H, n = u.shape
    N = M.shape[0]
    assert n <= N and k.shape[0] == H and k.shape[1] <= N
    kp = np.zeros((H, N))
    kp[:, :k.shape[1]] = k
    kf = kp @ M.T                                   # (H, N): row h = M k_h
    a = u * np.asarray(g_in, dtype=np.float64) if g_in is not None else u
    ap = np.zeros((B, H, N))
    ap[:, :, :n] = a
    uf = ap @ M.T
    f = np.linalg.solve(M, (kf[None] * uf).reshape(B * H, N).T).T.reshape(B, H, N)
    y = f.real[:, :, :n]
    if g_out is not None:
        y = y * np.asarray(g_out, dtype=np.float64)
    return y, f
