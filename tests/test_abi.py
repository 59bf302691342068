"""C-ABI checks that need no GPU: the library loads, exports what the header declares,
and rejects bad arguments before any device work."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2310_12109_amd", "libmonarch.so")
HEADER = os.path.join(ROOT, "include", "monarch.h")

EINVAL, ESHAPE, EDTYPE, EWORKSPACE = -1, -2, -3, -4


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        pytest.fail("libmonarch.so is not built; run __graft_entry__.build() first")
    from paper_2310_12109_amd import binding
    return binding.raw()


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(monarch_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = _declared_functions()
    assert len(names) >= 12
    for name in names:
        assert hasattr(lib, name), f"{name} declared in monarch.h but not exported"


def test_binding_lists_the_same_names(lib):
    from paper_2310_12109_amd import binding
    assert sorted(binding.EXPORTS) == _declared_functions()


@pytest.mark.parametrize("b,N", [(1, 1), (2, 6), (3, 6), (16, 256), (64, 2048), (32, 2048), (7, 49)])
def test_permutation_index_bit_exact_against_oracle(lib, b, N):
    out = np.empty(N, dtype=np.int32)
    assert lib.monarch_permutation_index(b, N, out.ctypes.data_as(ctypes.c_void_p)) == 0
    assert np.array_equal(out, oracle.perm(b, N))


def test_permutation_index_errors(lib):
    out = np.empty(8, dtype=np.int32)
    assert lib.monarch_permutation_index(2, 8, None) == EINVAL
    assert lib.monarch_permutation_index(3, 8, out.ctypes.data_as(ctypes.c_void_p)) == ESHAPE
    assert b"divide" in lib.monarch_last_error()


FAKE = 0x1000   # aligned, never dereferenced: every call below must fail before touching it


def test_matmul_rejects_bad_arguments(lib):
    f = lib.monarch_matmul
    assert f(None, FAKE, FAKE, FAKE, 4, 16, 16, 16, 16, 16, 16, 0, None, 0, None) == EINVAL
    assert f(FAKE, FAKE, FAKE, FAKE, 4, 16, 16, 16, 8, 16, 16, 0, None, 0, None) == ESHAPE   # d_mid mismatch
    assert f(FAKE, FAKE, FAKE, FAKE, 4, 0, 16, 16, 16, 16, 16, 0, None, 0, None) == ESHAPE
    assert f(FAKE, FAKE, FAKE, FAKE, 4, 16, 16, 16, 16, 16, 16, 2, None, 0, None) == EINVAL   # fp16 is taken: y aliases x
    assert f(FAKE, FAKE, FAKE, FAKE, 4, 16, 16, 16, 16, 16, 16, 9, None, 0, None) == EDTYPE
    assert f(FAKE + 4, FAKE, FAKE, FAKE * 2, 4, 16, 16, 16, 16, 16, 16, 0, None, 0, None) == EINVAL  # misaligned
    assert f(FAKE, FAKE * 4, FAKE * 8, FAKE, 4, 16, 16, 16, 16, 16, 16, 0, None, 0, None) == EINVAL  # y aliases x
    assert f(FAKE, FAKE, FAKE, FAKE, -1, 16, 16, 16, 16, 16, 16, 0, None, 0, None) == ESHAPE
    assert f(FAKE, FAKE, FAKE, FAKE * 64, 4, 256, 256, 256, 256, 256, 256, 0, None, 0, None) == ESHAPE  # too wide
    assert lib.monarch_strerror(ESHAPE) and lib.monarch_last_error()


def test_matmul_backward_rejects_bad_arguments(lib):
    f = lib.monarch_matmul_backward
    f.argtypes = [ctypes.c_void_p] * 7 + [ctypes.c_int64] + [ctypes.c_int] * 7 + [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    A, B, C, D, E, F, G = (FAKE * m for m in (1, 16, 32, 48, 64, 80, 96))   # 64 KB apart: no overlap at batch 4
    sq = (16, 16, 16, 16, 16, 16)
    assert f(None, B, C, D, E, F, G, 4, *sq, 0, None, 0, None) == EINVAL            # x missing
    assert f(A, B, C, None, E, F, G, 4, *sq, 0, None, 0, None) == EINVAL            # dy missing
    assert f(A, B, C, D, E, F, G, 4, 16, 16, 16, 8, 16, 16, 0, None, 0, None) == ESHAPE   # d_mid mismatch
    assert f(A, B, C, D, E, F, G, 4, *sq, 2, None, 0, None) == EDTYPE
    assert f(A, B, C, D, E, F, G, -1, *sq, 0, None, 0, None) == ESHAPE
    assert f(A + 4, B, C, D, E, F, G, 4, *sq, 0, None, 0, None) == EINVAL           # misaligned
    assert f(A, B, C, D, A, F, G, 4, *sq, 0, None, 0, None) == EINVAL               # dx aliases x
    assert f(A, B, C, D, E, B, G, 4, *sq, 0, None, 0, None) == EINVAL               # dR aliases R
    assert f(A, B, C, D, E, F, F, 4, *sq, 0, None, 0, None) == EINVAL               # dR aliases dL
    assert f(A, B, C, D, None, None, None, 4, *sq, 0, None, 0, None) == 0           # nothing asked for
    assert f(A, B, C, D, E, F, G, 4, 256, 256, 256, 256, 256, 256, 0, None, 0, None) == ESHAPE   # too wide


def test_matmul3_rejects_bad_arguments(lib):
    f = lib.monarch_matmul3
    f.argtypes = [ctypes.c_void_p] * 5 + [ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    x, B1, B2, B3, y = (FAKE * m for m in (1, 64, 128, 192, 256))   # 256 KB apart
    assert f(None, B1, B2, B3, y, 4, 8, 0, None) == EINVAL
    assert f(x, B1, B2, None, y, 4, 8, 0, None) == EINVAL
    assert f(x, B1, B2, B3, x, 4, 8, 0, None) == EINVAL        # y aliases x
    assert f(x + 4, B1, B2, B3, y, 4, 8, 0, None) == EINVAL    # misaligned
    assert f(x, B1, B2, B3, y, -1, 8, 0, None) == ESHAPE
    assert f(x, B1, B2, B3, y, 4, 17, 0, None) == ESHAPE       # b^3 beyond the on-chip tile
    assert f(x, B1, B2, B3, y, 4, 0, 0, None) == ESHAPE
    assert f(x, B1, B2, B3, y, 4, 8, 2, None) == EDTYPE
    assert f(None, None, None, None, None, 0, 8, 0, None) == 0
    g = lib.monarch_matmul3_backward
    g.argtypes = [ctypes.c_void_p] * 9 + [ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    dy, dx, d1, d2, d3 = (FAKE * m for m in (320, 384, 448, 512, 576))
    assert g(x, B1, B2, B3, None, dx, d1, d2, d3, 4, 8, 0, None) == EINVAL       # dy missing
    assert g(x, B1, B2, B3, dy, x, d1, d2, d3, 4, 8, 0, None) == EINVAL          # dx aliases x
    assert g(x, B1, B2, B3, dy, dx, B1, d2, d3, 4, 8, 0, None) == EINVAL         # dB1 aliases B1
    assert g(x, B1, B2, B3, dy, dx, d1, d1, d3, 4, 8, 0, None) == EINVAL         # dB1 aliases dB2
    assert g(x, B1, B2, B3, dy, dx, d1, d2, d3, 4, 17, 0, None) == ESHAPE
    assert g(x, B1, B2, B3, dy, None, None, None, None, 4, 8, 0, None) == 0      # nothing asked for


def test_mixer_rejects_bad_arguments(lib):
    f = lib.monarch_mixer
    f.argtypes = [ctypes.c_void_p] * 9 + [ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    u, K, gi, go, R1, L1, R2, L2, y = (FAKE * m for m in (1, 16, 32, 48, 64, 65, 66, 67, 80))   # >= 64 KB apart
    assert f(None, K, gi, go, R1, L1, R2, L2, y, 2, 4, 16, 0, None, 0, None) == EINVAL      # u missing
    assert f(u, K, gi, go, R1, None, R2, L2, y, 2, 4, 16, 0, None, 0, None) == EINVAL       # a factor missing
    assert f(u, K, None, None, R1, L1, R2, L2, None, 2, 4, 16, 0, None, 0, None) == EINVAL  # y missing
    assert f(u, K, gi, go, R1, L1, R2, L2, u, 2, 4, 16, 0, None, 0, None) == EINVAL         # y aliases u
    assert f(u, K, gi, go, R1, L1, R2, L2, go, 2, 4, 16, 0, None, 0, None) == EINVAL        # y aliases a gate
    assert f(u + 8, K, gi, go, R1, L1, R2, L2, y, 2, 4, 16, 0, None, 0, None) == EINVAL     # misaligned
    assert f(u, K, gi, go, R1, L1, R2, L2, y, -1, 4, 16, 0, None, 0, None) == ESHAPE
    assert f(u, K, gi, go, R1, L1, R2, L2, y, 2, 0, 16, 0, None, 0, None) == ESHAPE
    assert f(u, K, gi, go, R1, L1, R2, L2, y, 2, 4, 0, 0, None, 0, None) == ESHAPE
    assert f(u, K, gi, go, R1, L1, R2, L2, y, 2, 4, 256, 0, None, 0, None) == ESHAPE        # a row beyond LDS
    assert f(u, K, gi, go, R1, L1, R2, L2, y, 2, 4, 16, 2, None, 0, None) == EDTYPE
    assert f(None, None, None, None, None, None, None, None, None, 0, 4, 16, 0, None, 0, None) == 0   # nothing to do
    assert lib.monarch_mixer_workspace_bytes(8, 4, 16, 0) == 0


def test_mixer_backward_rejects_bad_arguments(lib):
    f = lib.monarch_mixer_backward
    f.argtypes = [ctypes.c_void_p] * 17 + [ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.monarch_mixer_backward_workspace_bytes.restype = ctypes.c_size_t
    lib.monarch_mixer_backward_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int]
    need = lib.monarch_mixer_backward_workspace_bytes(2, 4, 16, 0)
    assert need >= 5 * 2 * 4 * 256 * 4
    p = [FAKE * (64 * (i + 1)) for i in range(17)]      # 256 KB apart
    ws = FAKE * 4096

    def call(p=p, B=2, H=4, bs=16, dt=0, ws=ws, wsb=need):
        return f(*p, B, H, bs, dt, ws, wsb, None)

    def with_(i, v):
        q = list(p); q[i] = v
        return q
    assert call(with_(0, None)) == EINVAL                 # u missing
    assert call(with_(8, None)) == EINVAL                 # dy missing
    assert call(with_(2, None)) == EINVAL                 # dg_in asked for without g_in
    assert call(with_(9, p[0])) == EINVAL                 # du aliases u
    assert call(with_(13, p[4])) == EINVAL                # dR1 aliases R1
    assert call(with_(14, p[13])) == EINVAL               # dL1 aliases dR1
    assert call(with_(0, p[0] + 4)) == EINVAL             # misaligned
    assert call(ws=p[0]) == EINVAL                        # workspace over u
    assert call(wsb=need - 1) == EWORKSPACE
    assert call(ws=None) == EWORKSPACE
    assert call(B=-1) == ESHAPE
    assert call(H=0) == ESHAPE
    assert call(bs=0) == ESHAPE
    assert call(bs=200) == ESHAPE
    assert call(dt=9) == EDTYPE


def test_m2_layer_rejects_bad_arguments(lib):
    f = lib.monarch_m2_layer
    f.argtypes = ([ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_int] + [ctypes.c_void_p] * 12 +
                  [ctypes.c_float, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p])
    lib.monarch_m2_layer_workspace_bytes.restype = ctypes.c_size_t
    lib.monarch_m2_layer_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int]
    need = lib.monarch_m2_layer_workspace_bytes(2, 256, 256, 0)
    assert need >= 2 * 256 * 256 * 4
    x, y, ws = FAKE * 1024, FAKE * 2048, FAKE * 4096          # 4 MB apart
    p = [FAKE * (16 + i) for i in range(12)]

    def call(x=x, y=y, B=2, bn=16, bd=16, p=p, eps=1e-5, act=1, dt=0, ws=ws, wsb=need):
        return f(x, y, B, bn, bd, *p, eps, act, dt, ws, wsb, None)
    assert call(x=None) == EINVAL
    assert call(p=p[:5] + [None] + p[6:]) == EINVAL
    assert call(y=x) == EINVAL                   # y aliases x
    assert call(ws=x) == EINVAL                  # workspace aliases x
    assert call(x=x + 8) == EINVAL               # misaligned
    assert call(act=2) == EINVAL
    assert call(eps=-1.0) == EINVAL
    assert call(B=-1) == ESHAPE
    assert call(bn=0) == ESHAPE
    assert call(bd=200) == ESHAPE                # a row beyond LDS
    assert call(dt=9) == EDTYPE
    assert call(wsb=need - 1) == EWORKSPACE
    assert call(B=0) == 0


def test_blocky_rejects_bad_arguments(lib):
    lib.monarch_blocky_state_bytes.restype = ctypes.c_size_t
    lib.monarch_blocky_state_bytes.argtypes = [ctypes.c_int, ctypes.c_int]
    need = lib.monarch_blocky_state_bytes(4, 16)
    assert need >= 256 * 16 + 4 * 4096 * 8 + 4 * 256 * 8
    assert lib.monarch_blocky_state_bytes(4, 65) == 0
    off = (ctypes.c_size_t * 5)()
    lib.monarch_blocky_state_offsets.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_size_t)]
    assert lib.monarch_blocky_state_offsets(4, 16, off) == 0
    assert list(off) == sorted(off) and off[0] >= 256 * 16 and off[4] + 4 * 256 * 8 <= need
    assert all(o % 256 == 0 for o in off) and off[1] - off[0] >= 4096 * 8
    assert lib.monarch_blocky_state_offsets(4, 65, off) == ESHAPE
    assert lib.monarch_blocky_state_offsets(4, 16, None) == EINVAL
    p = lib.monarch_blocky_prepare
    p.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_int] * 4 + [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    Lt, Rt, k, st = FAKE, FAKE * 8, FAKE * 16, FAKE * 64
    assert p(None, Rt, k, 4, 128, 16, 1, st, need, None) == EINVAL
    assert p(Lt, Rt, k, 4, 128, 16, 1, None, need, None) == EINVAL
    assert p(Lt, Rt, k, 4, 128, 16, 2, st, need, None) == EINVAL            # mask flag
    assert p(Lt, Rt, k, 4, 128, 1, 1, st, need, None) == ESHAPE             # block size
    assert p(Lt, Rt, k, 4, 128, 65, 1, st, 1 << 40, None) == ESHAPE
    assert p(Lt, Rt, k, 4, 129, 16, 1, st, need, None) == ESHAPE            # more taps than the mask allows
    assert p(Lt, Rt, k, 4, 257, 16, 0, st, need, None) == ESHAPE            # more taps than N
    assert p(Lt, Rt, k, 4, 128, 16, 1, st, need - 1, None) == EWORKSPACE
    assert p(Lt, Rt, k, 4, 128, 16, 1, Lt, need, None) == EINVAL            # state over the coefficients
    c = lib.monarch_blocky_conv
    c.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int64] + [ctypes.c_int] * 4 + [ctypes.c_void_p]
    u, gi, go, y = FAKE * 128, FAKE * 160, FAKE * 192, FAKE * 224
    assert c(None, gi, go, st, need, y, 2, 4, 128, 16, 0, None) == EINVAL
    assert c(u, gi, go, None, need, y, 2, 4, 128, 16, 0, None) == EINVAL
    assert c(u, gi, go, st, need - 1, y, 2, 4, 128, 16, 0, None) == EWORKSPACE
    assert c(u, gi, go, st, need, u, 2, 4, 128, 16, 0, None) == EINVAL       # y aliases u
    assert c(u, gi, go, st, need, y, 2, 4, 257, 16, 0, None) == ESHAPE       # n beyond N
    assert c(u, gi, go, st, need, y, 2, 0, 128, 16, 0, None) == ESHAPE
    assert c(u, gi, go, st, need, y, 2, 4, 128, 16, 2, None) == EDTYPE
    assert c(u, gi, go, st, need, y, 0, 4, 128, 16, 0, None) == 0            # nothing to do


def test_fft_rejects_bad_arguments(lib):
    fac = (ctypes.c_int * 3)(64, 32, 1)
    bad = (ctypes.c_int * 2)(64, 31)
    one = (ctypes.c_int * 2)(2048, 1)
    f = lib.monarch_fft
    assert f(FAKE, FAKE * 1024, 4, 2048, fac, 1, 1, 0, FAKE, 1 << 30, None) == ESHAPE       # nf = 1
    assert f(FAKE, FAKE * 1024, 4, 2048, bad, 2, 1, 0, FAKE, 1 << 30, None) == ESHAPE       # product
    assert f(FAKE, FAKE * 1024, 4, 2048, one, 2, 1, 0, FAKE, 1 << 30, None) == ESHAPE       # factor < 2
    assert f(FAKE, FAKE * 1024, 4, 2048, None, 2, 1, 0, FAKE, 1 << 30, None) == EINVAL
    assert f(FAKE, FAKE * 1024, 4, 2048, fac, 2, 1, 0, None, 0, None) == EWORKSPACE
    assert f(FAKE, FAKE * 1024, 4, 2048, fac, 2, 1, 0, FAKE, 100, None) == EWORKSPACE
    assert f(FAKE, None, 4, 2048, fac, 2, 1, 0, FAKE, 1 << 30, None) == EINVAL
    assert f(FAKE, FAKE * 1024, 4, 2048, fac, 2, 7, 0, FAKE, 1 << 30, None) == EINVAL       # real flag
    assert lib.monarch_ifft(FAKE, FAKE * 1024, 4, 2048, fac, 2, 1, 9, FAKE, 1 << 30, None) == EDTYPE
    need = lib.monarch_fft_workspace_bytes(4, 2048, fac, 2, 0)
    assert need >= 4 * 2048 * 8


def test_conv_rejects_bad_arguments(lib):
    fac = (ctypes.c_int * 2)(64, 32)
    f = lib.monarch_causal_conv
    big = 1 << 40
    # rows of 1022 elements have no fused kernel: every accepted call would need the workspace, and the calls below
    # all fail before any launch (the pointers are fake)
    args = dict(B=8, H=4, n=1022, klen=1022, nfft=2048)

    def call(u=FAKE, k=FAKE * 2, y=FAKE * 1 << 20, causal=1, dt=0, ws=FAKE * 1 << 24, wsb=big, **kw):
        a = dict(args); a.update(kw)
        return f(u, k, None, None, y, a["B"], a["H"], a["n"], a["klen"], a["nfft"], fac, 2, causal, dt, ws, wsb, None)

    assert call(u=None) == EINVAL
    assert call(n=2049) == ESHAPE
    assert call(n=1025, klen=1025) == ESHAPE            # would wrap around
    assert call(klen=2000) == ESHAPE                    # causal kernel longer than the sequence
    assert call(klen=4096, causal=0) == ESHAPE
    assert call(causal=2) == EINVAL
    assert call(dt=9) == EDTYPE
    assert call(ws=None, wsb=0) == EWORKSPACE
    assert call(wsb=64) == EWORKSPACE
    assert call(y=FAKE) == EINVAL                        # y aliases u
    assert lib.monarch_causal_conv_workspace_bytes(8, 4, 1022, 1022, 2048, fac, 2, 0) > 0
    for dt in (0, 1, 2):    # the fused 64 x 32 kernels (fp32, bf16, fp16) need none
        assert lib.monarch_causal_conv_workspace_bytes(8, 4, 1024, 1024, 2048, fac, 2, dt) == 0


def test_mlp_rejects_bad_arguments(lib):
    f = lib.monarch_mlp
    Y = FAKE << 20

    def call(x=FAKE, y=Y, tokens=16, d=768, dh=3072, nb=4, order=1, w1l=None, w2l=None, act=2, dt=1,
             ws=FAKE << 24, wsb=1 << 40, mid1=0, mid2=0):
        return f(x, y, tokens, d, dh, nb, order, FAKE, w1l, None, FAKE, w2l, None, mid1, mid2, act, dt, ws, wsb, None)

    assert call(x=None) == EINVAL
    assert call(nb=5) == ESHAPE
    assert call(order=3) == ESHAPE
    assert call(act=5) == EINVAL
    assert call(order=2) == EINVAL                       # order 2 without the L factors
    assert call(order=1, w1l=FAKE) == EINVAL
    assert call(order=2, w1l=FAKE, w2l=FAKE, mid1=770) == ESHAPE
    assert call(dt=9) == EDTYPE
    # order 2 keeps the hidden activations in the workspace (the fused order-1 kernel needs none)
    assert call(order=2, w1l=FAKE, w2l=FAKE, ws=None, wsb=0) == EWORKSPACE
    assert call(y=FAKE) == EINVAL
    # order 2, bf16: the two d_mid-wide intermediates; fp32: the hidden activations
    assert lib.monarch_mlp_workspace_bytes(16, 768, 3072, 4, 2, 0, 0, 1) >= 2 * 16 * 768 * 2
    assert lib.monarch_mlp_workspace_bytes(16, 768, 3072, 4, 2, 0, 0, 0) >= 16 * 3072 * 4
