"""CPU oracle for the general (learned, real) order-3 Monarch product and its gradients (Sec. 3.1 and the
appendix definition of order-p Monarch matrices, p = 3).

TEST INFRASTRUCTURE ONLY.  Plain numpy, float64.  N = b^3; three block-diagonal factors B1, B2, B3, each
[b*b blocks][b][b], B1 applied first:  M = P^R B3 P_(b,b^2,N) B2 P_(b^2,b^3,N) B1 P^R  (the dense form of this
product is oracle.monarch3_dense, against which the steps below are pinned).  With the input index
j = j2 b^2 + j1 b + j0 and the output index m = m2 b^2 + m1 b + m0 the permutations say which sub-index each
factor consumes and how its blocks are numbered (block (p, q) is block p b + q):
    t1[(j0,j1), m0] = sum_j2 B1[(j0,j1)][m0, j2] x[j2, j1, j0]
    t2[(m0,j0), m1] = sum_j1 B2[(m0,j0)][m1, j1] t1[(j0,j1), m0]
    y[m2, m1, m0]   = sum_j0 B3[(m0,m1)][m2, j0] t2[(m0,j0), m1]
"""
import numpy as np


def _blocks(B, b):
    return np.asarray(B, dtype=np.float64).reshape(b, b, b, b)   # [p][q][row][col]


def matmul3(x, B1, B2, B3):
    """y[v, :] = M x[v, :] by the three steps above; x: (batch, b^3)."""
    b = B1.shape[-1]
    X = np.asarray(x, dtype=np.float64).reshape(-1, b, b, b)          # [v][j2][j1][j0]
    t1 = np.einsum("pqrc,vcqp->vpqr", _blocks(B1, b), X)              # [v][j0][j1][m0]
    t2 = np.einsum("pqrc,vqcp->vpqr", _blocks(B2, b), t1)             # [v][m0][j0][m1]:  B2[(m0,j0)][m1,j1] t1[j0][j1][m0]
    y = np.einsum("pqrc,vpcq->vrqp", _blocks(B3, b), t2)              # [v][m2][m1][m0]:  B3[(m0,m1)][m2,j0] t2[m0][j0][m1]
    return y.reshape(-1, b ** 3)


def matmul3_backward(x, B1, B2, B3, dy):
    """(dx, dB1, dB2, dB3) of S = sum_v <dy[v], M x[v]>: the adjoint of each of the three steps, last step first
    (the paper states the forward product only; this is the chain rule through it)."""
    b = B1.shape[-1]
    X = np.asarray(x, dtype=np.float64).reshape(-1, b, b, b)
    G = np.asarray(dy, dtype=np.float64).reshape(-1, b, b, b)          # [v][m2][m1][m0]
    W1, W2, W3 = _blocks(B1, b), _blocks(B2, b), _blocks(B3, b)
    t1 = np.einsum("pqrc,vcqp->vpqr", W1, X)
    t2 = np.einsum("pqrc,vqcp->vpqr", W2, t1)
    dB3 = np.einsum("vrqp,vpcq->pqrc", G, t2)                          # [(m0,m1)][m2][j0]
    g2 = np.einsum("pqrc,vrqp->vpcq", W3, G)                           # [v][m0][j0][m1]
    dB2 = np.einsum("vpqr,vqcp->pqrc", g2, t1)                         # [(m0,j0)][m1][j1]
    g1 = np.einsum("pqrc,vpqr->vqcp", W2, g2)                          # [v][j0][j1][m0]
    dB1 = np.einsum("vpqr,vcqp->pqrc", g1, X)                          # [(j0,j1)][m0][j2]
    dx = np.einsum("pqrc,vpqr->vcqp", W1, g1)                          # [v][j2][j1][j0]
    shape = (b * b, b, b)
    return dx.reshape(-1, b ** 3), dB1.reshape(shape), dB2.reshape(shape), dB3.reshape(shape)
