"""CPU oracle for the general (learned) order-p Monarch product and its gradients (Sec. 3.1 and the appendix
definition of the p-variate Monarch matrix with the lemma that numbers the blocks of its factors).

TEST INFRASTRUCTURE ONLY.  Plain numpy, float64 (complex128 when a factor is complex: the DFT pins).  N = b^p;
B: (p, b^(p-1), b, b), B[0] applied first.  The matrix is the product written out,

    M = P^R  BD(B_p)  P_(b, b^2, N)  BD(B_(p-1))  P_(b^2, b^3, N)  ...  BD(B_2)  P_(b^(p-1), b^p, N)  BD(B_1)  P^R

with BD(.) the block-diagonal matrix of a factor, P_(b', M, N) = diag of N / M copies of the permutation P_(b', M)
((P x)[i] = x[sigma[i]], sigma[i1 b' + i0] = i0 (M / b') + i1) and P^R the reversal of the p base-b digits of an index.
With these permutations the blocks of factor s are numbered by the output digits already produced (most significant)
followed by the input digits not yet consumed, the numbering the lemma prescribes; p = 3 is oracle.monarch3_dense.
"""
import numpy as np


def sigma(bp, Mp, N):
    """Index vector of P_(bp, Mp, N): (P x)[i] = x[sigma[i]]."""
    assert Mp % bp == 0 and N % Mp == 0
    q = Mp // bp
    i = np.arange(Mp)
    one = (i % bp) * q + i // bp
    return (np.arange(N // Mp)[:, None] * Mp + one[None, :]).reshape(N)


def reversal(b, p):
    """Index vector of P^R: position (i_(p-1) .. i_0) reads position (i_0 .. i_(p-1))."""
    N = b ** p
    i = np.arange(N)
    out = np.zeros(N, dtype=np.int64)
    for _ in range(p):
        out = out * b + i % b
        i = i // b
    return out


def _bd(Bs, A):
    """BD(Bs) A for the block-diagonal matrix of Bs: (nb, b, b) and a dense A with nb b rows."""
    nb, b, _ = Bs.shape
    return np.einsum("krc,kcn->krn", Bs, A.reshape(nb, b, -1)).reshape(nb * b, -1)


def _shape(B):
    B = np.asarray(B)
    B = B.astype(np.complex128 if np.iscomplexobj(B) else np.float64)
    p, nb, b, b2 = B.shape
    assert b == b2 and nb == b ** (p - 1) and p >= 2
    return B, p, b, b ** p


def _prefixes(B):
    """C[s] for s = 1 .. p: the dense matrix of everything applied before factor s (C[1] = P^R); C[p + 1] = M."""
    B, p, b, N = _shape(B)
    A = np.eye(N, dtype=B.dtype)[reversal(b, p)]            # P^R
    C = [None, A]
    for s in range(1, p + 1):
        A = _bd(B[s - 1], A)
        A = A[sigma(b ** (p - s), b ** (p - s + 1), N)] if s < p else A[reversal(b, p)]
        C.append(A)
    return C


def orderp_dense(B):
    """The dense N x N matrix M of the product above."""
    return _prefixes(B)[-1]


def matmulp(x, B):
    """y[v, :] = M x[v, :]; x: (batch, b^p)."""
    return np.asarray(x) @ orderp_dense(B).T


def matmulp_backward(x, B, dy):
    """(dx, dB) of S = sum_v <dy[v], M x[v]> (the paper states the forward product only; this is the chain rule through
    it): with M = A_s BD(B_s) C_s for every factor s, dx = M^T dy and dB_s[k][r, c] = sum_v (A_s^T dy[v])[k b + r]
    (C_s x[v])[k b + c]."""
    B, p, b, N = _shape(B)
    x, dy = np.asarray(x, dtype=np.float64), np.asarray(dy, dtype=np.float64)
    C = _prefixes(B)
    # suffixes: S[s] = everything applied after factor s (S[p] = P^R), built from the last factor down
    S = [None] * (p + 1)
    S[p] = np.eye(N)[reversal(b, p)]
    for s in range(p - 1, 0, -1):
        # after factor s come P_(b^(p-s), b^(p-s+1), N), then BD(B_(s+1)), then S[s + 1]
        Pm = np.eye(N)[sigma(b ** (p - s), b ** (p - s + 1), N)]
        S[s] = S[s + 1] @ _bd(B[s], Pm)
    dB = np.empty((p, b ** (p - 1), b, b))
    for s in range(1, p + 1):
        X = (x @ C[s].T).reshape(-1, b ** (p - 1), b)            # C_s x
        G = (dy @ S[s]).reshape(-1, b ** (p - 1), b)             # A_s^T dy
        dB[s - 1] = np.einsum("vkr,vkc->krc", G, X)
    return dy @ C[-1], dB
