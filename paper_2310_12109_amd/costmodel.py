"""Host-side cost model: algorithmic bytes and FLOPs of the hot path (used by the benchmark)."""
import math


def paper_dense_flops(N, d=768):
    """Dense N x N matmul applied to d columns: the 'Dense Matmul' row of the paper's Table 2."""
    return 2.0 * N * N * d


def paper_m2_flops(N, d=768):
    """M (K o M X) with two real order-2 Monarch products per column, b = sqrt(N): Table 2's M2 row."""
    return 8.0 * N ** 1.5 * d


def monarch_matmul_flops(nbR, r_out, r_in, nbL, l_out, l_in):
    """Real order-2 Monarch product, per vector (Sec. 3.1): 2 FLOP per stored weight."""
    return 2.0 * (nbR * r_out * r_in + nbL * l_out * l_in)


def conv_algorithmic_bytes(B, H, n, klen, dtype_bytes, gates=2):
    """Minimum HBM traffic of one gated convolution: u and y, the gate streams, and k once."""
    return (2 + gates) * B * H * n * dtype_bytes + H * klen * dtype_bytes


def conv_executed_flops(B, H, factors):
    """FLOPs the convolution kernels actually issue, for two or three factors f0, f1[, f2] (N their product):
    two real rows share one complex transform (two batch entries of a channel; with B = 1 two neighbouring
    channels, the kernels paired alike), the zero-padded half of the first factor's input and the discarded
    half of its output in the inverse are skipped, and a real kernel row costs half a complex one in the first
    factor.  A complex DFT factor of size f over N points is four real GEMMs: 8 N f."""
    N = 1
    for f in factors:
        N *= f
    f0, rest = factors[0], sum(factors[1:])
    diagonals = 6.0 * N * (len(factors) - 1)
    row_forward = 4.0 * N * f0 + 8.0 * N * rest + diagonals             # complex row, half of the input zero
    row_inverse = 8.0 * N * rest + 4.0 * N * f0 + diagonals + 6.0 * N   # times k_f; half of the output dropped
    if B == 1 and H >= 2:
        crows = math.ceil(H / 2)
        return crows * (2 * row_forward + row_inverse)
    kernel_row = 2.0 * N * f0 + 8.0 * N * rest + diagonals              # real input
    return math.ceil(B / 2) * H * (row_forward + row_inverse) + H * kernel_row


def conv_textbook_flops(B, H, factors):
    """The same convolution with every stage complex and nothing skipped (for comparison)."""
    N = 1
    for f in factors:
        N *= f
    per_transform = sum(8.0 * N * f for f in factors) + 6.0 * N * (len(factors) - 1)
    return B * H * (2 * per_transform + 6.0 * N) + H * per_transform


def mlp_flops(tokens, d, d_hidden, nb, order, mid1=0, mid2=0):
    if order == 1:
        per = 2.0 * (d_hidden * d / nb) * 2
    else:
        mid1 = mid1 or d
        mid2 = mid2 or d
        per = 2.0 * (mid1 * d + d_hidden * mid1 + mid2 * d_hidden + d * mid2) / nb
    return tokens * per


def mlp_algorithmic_bytes(tokens, d, d_hidden, nb, order, dtype_bytes=2, mid1=0, mid2=0):
    if order == 1:
        w = 2 * d * d_hidden / nb
    else:
        mid1 = mid1 or d
        mid2 = mid2 or d
        w = (mid1 * d + d_hidden * mid1 + mid2 * d_hidden + d * mid2) / nb
    return (2 * tokens * d + w + d + d_hidden) * dtype_bytes
