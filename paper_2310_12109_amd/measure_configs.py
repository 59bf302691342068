"""Times every configuration of the hot path through the binding and prints one line per case:
`python -m paper_2310_12109_amd.measure_configs [c1 copy c1b mixerb mm3 mixer layer blocky c2 fft c3a c3b c4 c5a c5b]`.

Inputs are random tensors of each configuration's shapes and dtypes, already resident in HBM.  Every case
rotates over enough distinct buffer sets to exceed 512 MB (at most 24 sets), so that the 256 MB Infinity
Cache cannot serve a working set that is smaller than it; time = HIP events around `reps` back-to-back
launches (replayed from a HIP graph), divided by their number.  Rates are algorithmic: bytes every implementation must move and the
textbook FLOPs of the method (costmodel.py), over the measured time.
"""
import sys

import torch

from . import binding, costmodel

HBM_PEAK_GBS = 8000.0


def _sets(make, bytes_per_set):
    n = max(1, min(24, int(512e6 // max(bytes_per_set, 1)) + 1))
    return [make() for _ in range(n)]


def _time(calls, reps):
    """One pass over every buffer set is captured into a HIP graph and replayed, so that a kernel of a
    few microseconds is not timed at the rate the interpreter can launch it."""
    for c in calls:   # warm-up
        c()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for c in calls:
            c()
    graph.replay()
    torch.cuda.synchronize()
    rounds = max(1, reps // len(calls))
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(rounds):
        graph.replay()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) * 1e3 / (rounds * len(calls))   # microseconds per call


def _rnd(*shape, dt=torch.bfloat16, scale=1.0):
    return (torch.randn(*shape, device="cuda") * scale).to(dt)


def _report(name, us, nbytes, flops, nsets):
    gbs = nbytes / us / 1e3
    print(f"{name:42s} {us:9.1f} us  {gbs:8.1f} GB/s ({gbs / HBM_PEAK_GBS:5.3f} of HBM)  {flops / us / 1e6:8.1f} TFLOP/s  "
          f"[{nsets} buffer sets]", flush=True)


def matmul_c1(batch, reps, dt=torch.float32):
    es = 4 if dt == torch.float32 else 2
    nbytes = (2 * batch * 256 + 2 * 16 * 256) * es
    R, L = _rnd(16, 16, 16, dt=dt, scale=.25), _rnd(16, 16, 16, dt=dt, scale=.25)

    def make():
        x = _rnd(batch, 256, dt=dt)
        y = torch.empty_like(x)
        return lambda: binding.monarch_matmul(x, R, L, out=y)
    calls = _sets(make, nbytes)
    _report(f"c1 matmul {'fp32' if es == 4 else 'bf16'} 16x16 blocks, batch {batch}", _time(calls, reps), nbytes, batch * 4 * 256 * 16, len(calls))


def plain_copy(mbytes, reps):
    """A device-to-device copy of `mbytes` MB (read + written: twice that) with torch's copy kernel: what this
    machine's memory system gives a kernel with no arithmetic, as a yardstick beside the 8 TB/s of the data sheet."""
    n = int(mbytes * 1e6) // 16 * 16

    def make():
        a = torch.empty(n, dtype=torch.uint8, device="cuda")
        b = torch.empty(n, dtype=torch.uint8, device="cuda")
        return lambda: b.copy_(a)
    calls = _sets(make, 2 * n)
    _report(f"plain copy, {2 * n / 1e6:.0f} MB moved", _time(calls, reps), 2 * n, 0, len(calls))


def matmul_backward_c1(batch, reps, dt=torch.float32):
    """Gradients of the config-1 product: reads x and dy, writes dx (3 rows of 256 per vector); dR, dL are 32 KB."""
    es = 4 if dt == torch.float32 else 2
    nbytes = 3 * batch * 256 * es + 2 * 16 * 256 * (es + 4)
    R, L = _rnd(16, 16, 16, dt=dt, scale=.25), _rnd(16, 16, 16, dt=dt, scale=.25)

    def make():
        x, dy = _rnd(batch, 256, dt=dt), _rnd(batch, 256, dt=dt)
        return lambda: binding.monarch_matmul_backward(x, R, L, dy)
    calls = _sets(make, nbytes)
    # 5 block-diagonal products of 2 * 256 * 16 FLOP per vector (t1, g2, g0, dR, dL)
    _report(f"c1 matmul backward {'fp32' if es == 4 else 'bf16'}, batch {batch}", _time(calls, reps), nbytes, batch * 5 * 2 * 256 * 16, len(calls))


def mixer(B, H, reps, dt=torch.float32):
    """Learned-Monarch sequence mixer at N = 256: u, both gates read and y written (4 rows of 256 per row)."""
    rows = B * H
    es = 4 if dt == torch.float32 else 2
    nbytes = (4 * rows * 256 + H * 256 + 4 * 16 * 256) * es
    K = _rnd(H, 256, dt=dt)
    f = [_rnd(16, 16, 16, dt=dt, scale=.25) for _ in range(4)]

    def make():
        u, gi, go = (_rnd(B, H, 256, dt=dt) for _ in range(3))
        y = torch.empty_like(u)
        return lambda: binding.monarch_mixer(u, K, gi, go, *f, out=y)
    calls = _sets(make, nbytes)
    # four block-diagonal products of 2 * 256 * 16 FLOP per row
    _report(f"mixer {'fp32' if es == 4 else 'bf16'} N=256, B={B} H={H}", _time(calls, reps), nbytes, rows * 4 * 2 * 256 * 16, len(calls))


def matmul3(b, batch, reps):
    """General order-3 Monarch product and its gradients, fp32: 2 N floats per row forward, 3 N backward."""
    N = b ** 3
    f = [_rnd(b * b, b, b, dt=torch.float32, scale=b ** -0.5) for _ in range(3)]

    def make_fwd():
        x = _rnd(batch, N, dt=torch.float32)
        y = torch.empty_like(x)
        return lambda: binding.monarch_matmul3(x, *f, out=y)

    def make_bwd():
        x, dy = _rnd(batch, N, dt=torch.float32), _rnd(batch, N, dt=torch.float32)
        return lambda: binding.monarch_matmul3_backward(x, *f, dy)
    nb = 2 * batch * N * 4 + 3 * N * b * 4
    calls = _sets(make_fwd, nb)
    _report(f"order-3 matmul fp32 b={b} N={N}, batch {batch}", _time(calls, reps), nb, batch * 3 * 2 * N * b, len(calls))
    nb = 3 * batch * N * 4 + 6 * N * b * 4
    calls = _sets(make_bwd, nb)
    _report(f"order-3 backward fp32 b={b} N={N}, batch {batch}", _time(calls, reps), nb, batch * 8 * 2 * N * b, len(calls))


def m2_layer(B, reps, dt=torch.float32):
    """The basic M2 layer at n = d = 256: x read, X~ written and read, y written (4 passes over B n d elements)."""
    from . import workloads
    w = workloads.m2_layer_inputs(1, 16, 16, seed=0)
    par = {k: torch.from_numpy(v).cuda().to(dt) for k, v in w.items() if k != "x"}
    es = 4 if dt == torch.float32 else 2
    seq, dim = [par[k] for k in ("R1", "L1", "R2", "L2")], [par[k] for k in ("R3", "L3", "R4", "L4")]
    nbytes = (4 * B * 256 * 256 + 2 * 256 * 256) * es
    ws = torch.empty(binding.monarch_m2_layer_workspace_bytes(B, 256, 256, binding.F32 if es == 4 else binding.BF16),
                     dtype=torch.uint8, device="cuda")

    def make():
        x = _rnd(B, 256, 256, dt=dt)
        y = torch.empty_like(x)
        return lambda: binding.monarch_m2_layer(x, seq, par["n_kernel"], dim, par["d_kernel"], par["gamma"], par["beta"],
                                                ws=ws, out=y)
    calls = _sets(make, nbytes)
    # two mixers of four block-diagonal products each: 8 * 2 * 256 * 16 FLOP per row of 256
    _report(f"m2 layer {'fp32' if es == 4 else 'bf16'} n=256 d=256, B={B}", _time(calls, reps), nbytes, B * 2 * 256 * 8 * 2 * 256 * 16, len(calls))


def blocky(B, H, reps, dt=torch.float32):
    """Causal convolution with a polynomial-parameterised Monarch matrix, N = 256, n = 128: u and both gates
    read, y written; 704 complex-arithmetic MFMAs of 2048 FLOP per 16 rows."""
    from . import workloads
    rows, n = B * H, 128
    es = 4 if dt == torch.float32 else 2
    nbytes = 4 * rows * n * es + H * 256 * 8 + 4 * 4096 * 8
    w = workloads.blocky_inputs(1, H, n, 16, seed=0)
    par = [torch.from_numpy(w[k]).cuda() for k in ("Lt", "Rt", "k")]
    state = binding.monarch_blocky_prepare(*par, mask=True)

    def make():
        u, gi, go = (_rnd(B, H, n, dt=dt) for _ in range(3))
        y = torch.empty_like(u)
        return lambda: binding.monarch_blocky_conv(u, gi, go, state, 16, out=y)
    calls = _sets(make, nbytes)
    _report(f"blocky conv {'fp32' if es == 4 else 'bf16'} N=256 n=128, B={B} H={H}", _time(calls, reps), nbytes, rows / 16 * 704 * 2048, len(calls))
    if es == 4 and B <= 8:
        t = _time([lambda: binding.monarch_blocky_prepare(*par, mask=True, state=state)], 20)
        print(f"blocky prepare (factors, blockwise inverses, {H} kernels transformed) {t:9.1f} us", flush=True)


def mixer_backward(B, H, reps, dt=torch.float32):
    """Gradients of the learned-Monarch mixer at N = 256: u, gates, dy read; du, dg_in, dg_out written (7 arrays)."""
    rows = B * H
    es = 4 if dt == torch.float32 else 2
    nbytes = 7 * rows * 256 * es
    K = _rnd(H, 256, dt=dt)
    f = [_rnd(16, 16, 16, dt=dt, scale=.25) for _ in range(4)]
    ws = torch.empty(binding.raw().monarch_mixer_backward_workspace_bytes(B, H, 16, binding.F32 if es == 4 else binding.BF16),
                     dtype=torch.uint8, device="cuda")

    def make():
        u, gi, go, dy = (_rnd(B, H, 256, dt=dt) for _ in range(4))
        return lambda: binding.monarch_mixer_backward(u, K, gi, go, *f, dy, ws=ws)
    calls = _sets(make, nbytes)
    # forward again (2 products of 2 factors) and two gradient calls of 5 families each
    _report(f"mixer backward {'fp32' if es == 4 else 'bf16'} N=256, B={B} H={H}", _time(calls, reps), nbytes,
            rows * 14 * 2 * 256 * 16, len(calls))


def conv(name, B, H, n, factors, dt, reps):
    es = 2 if dt == torch.bfloat16 else 4
    code = binding.BF16 if dt == torch.bfloat16 else binding.F32
    nbytes = costmodel.conv_algorithmic_bytes(B, H, n, n, es)
    ws = torch.empty(max(16, binding.monarch_causal_conv_workspace_bytes(B, H, n, n, factors, code)), dtype=torch.uint8, device="cuda")

    def make():
        u, gi, go = _rnd(B, H, n, dt=dt), _rnd(B, H, n, dt=dt), _rnd(B, H, n, dt=dt)
        k = _rnd(H, n, dt=dt, scale=.1)
        y = torch.empty_like(u)
        return lambda: binding.monarch_causal_conv(u, k, gi, go, factors, ws=ws, out=y)
    calls = _sets(make, nbytes)
    _report(name, _time(calls, reps), nbytes, costmodel.conv_textbook_flops(B, H, factors), len(calls))


def fft(name, rows, factors, dt, reps):
    """Forward real-input transform and its inverse (complex spectrum, fp32 pairs, natural order)."""
    N = 1
    for f in factors:
        N *= f
    es = 2 if dt == torch.bfloat16 else 4
    nbytes = rows * N * (es + 8)
    flops = 0   # (the transforms are reported by their traffic only)

    def make_fwd():
        x = _rnd(rows, N, dt=dt)
        X = torch.empty((rows, N, 2), dtype=torch.float32, device="cuda")
        ws = torch.empty(max(16, binding.monarch_fft_workspace_bytes(rows, N, factors, binding.BF16 if dt == torch.bfloat16 else binding.F32)),
                         dtype=torch.uint8, device="cuda")
        return lambda: binding.monarch_fft(x, factors, True, ws=ws, out=X)

    def make_inv():
        X = torch.randn((rows, N, 2), dtype=torch.float32, device="cuda")
        x = torch.empty((rows, N), dtype=dt, device="cuda")
        ws = torch.empty(max(16, binding.monarch_fft_workspace_bytes(rows, N, factors, binding.BF16 if dt == torch.bfloat16 else binding.F32)),
                         dtype=torch.uint8, device="cuda")
        return lambda: binding.monarch_ifft(X, factors, True, dtype=dt, ws=ws, out=x)
    calls = _sets(make_fwd, 2 * nbytes)
    _report(name + " forward", _time(calls, reps), nbytes, flops, len(calls))
    calls = _sets(make_inv, 2 * nbytes)
    _report(name + " inverse", _time(calls, reps), nbytes, flops, len(calls))


def mlp(name, tokens, d, dh, nb, order, reps):
    nbytes = costmodel.mlp_algorithmic_bytes(tokens, d, dh, nb, order)
    std = 0.02
    if order == 1:
        w = dict(W1_R=_rnd(nb, dh // nb, d // nb, scale=std), W1_L=None, W2_R=_rnd(nb, d // nb, dh // nb, scale=std), W2_L=None)
    else:
        w = dict(W1_R=_rnd(nb, d // nb, d // nb, scale=std), W1_L=_rnd(nb, dh // nb, d // nb, scale=std),
                 W2_R=_rnd(nb, d // nb, dh // nb, scale=std), W2_L=_rnd(nb, d // nb, d // nb, scale=std))
    b1, b2 = _rnd(dh, scale=std), _rnd(d, scale=std)
    ws = torch.empty(max(16, binding.monarch_mlp_workspace_bytes(tokens, d, dh, nb, order)), dtype=torch.uint8, device="cuda")

    def make():
        x = _rnd(tokens, d)
        y = torch.empty_like(x)
        return lambda: binding.monarch_mlp(x, w["W1_R"], w["W1_L"], b1, w["W2_R"], w["W2_L"], b2, nb, order, 2, dh, ws=ws, out=y)
    calls = _sets(make, nbytes)
    _report(name, _time(calls, reps), nbytes, costmodel.mlp_flops(tokens, d, dh, nb, order), len(calls))


def main():
    only = sys.argv[1:]

    def want(name):
        return not only or name in only
    torch.manual_seed(0)
    if want("c1"):
        matmul_c1(64, 200)
        matmul_c1(1 << 20, 10)
        matmul_c1(1 << 20, 10, torch.bfloat16)
    if want("copy"):
        for mb in (12.6, 25.2, 50.4, 201, 805):
            plain_copy(mb, 100 if mb < 100 else 20)
    if want("c1b"):
        matmul_backward_c1(64, 100)
        matmul_backward_c1(1 << 20, 5)
        matmul_backward_c1(1 << 20, 5, torch.bfloat16)
    if want("mixer"):
        mixer(8, 768, 100)
        mixer(1024, 768, 5)
        mixer(8, 768, 100, torch.bfloat16)
        mixer(1024, 768, 5, torch.bfloat16)
    if want("mixerb"):
        mixer_backward(8, 768, 50)
        mixer_backward(256, 768, 5)
        mixer_backward(256, 768, 5, torch.bfloat16)
    if want("mm3"):
        matmul3(8, 16384, 10)
        matmul3(16, 4096, 10)
        matmul3(16, 65536, 2)
    if want("layer"):
        m2_layer(32, 50)
        m2_layer(2048, 5)
        m2_layer(2048, 5, torch.bfloat16)
    if want("blocky"):
        blocky(8, 768, 100)
        blocky(1024, 768, 5)
        blocky(1024, 768, 5, torch.bfloat16)
    if want("c2"):
        conv("c2 conv bf16 B=8 H=768 n=1024 64x32", 8, 768, 1024, (64, 32), torch.bfloat16, 200)
        conv("c2 conv fp32 B=8 H=768 n=1024 64x32", 8, 768, 1024, (64, 32), torch.float32, 50)
    if want("fft"):
        fft("fft bf16 real, 6144 rows of 2048 = 64x32", 6144, (64, 32), torch.bfloat16, 50)
        fft("fft fp32 real, 6144 rows of 2048 = 64x32", 6144, (64, 32), torch.float32, 30)
        fft("fft bf16 real, 1536 rows of 16384 = 128x128", 1536, (128, 128), torch.bfloat16, 20)
    if want("c3a"):
        conv("c3a conv bf16 B=32 H=768 n=128 16x16", 32, 768, 128, (16, 16), torch.bfloat16, 200)
    if want("c3b"):
        mlp("c3b mlp bf16 4096x768->3072 nb=4 order 1", 4096, 768, 3072, 4, 1, 100)
        mlp("c3b mlp bf16 4096x768->3072 nb=4 order 2", 4096, 768, 3072, 4, 2, 100)
    if want("c4"):
        conv("c4 conv bf16 B=4 H=768 n=8192 128x128", 4, 768, 8192, (128, 128), torch.bfloat16, 20)
    if want("c5a"):
        conv("c5a conv bf16 B=1 H=256 n=131072 64^3", 1, 256, 131072, (64, 64, 64), torch.bfloat16, 10)
    if want("c5b"):
        mlp("c5b mlp bf16 65536x1024->4096 nb=16 order 1", 65536, 1024, 4096, 16, 1, 20)
        mlp("c5b mlp bf16 65536x1024->4096 nb=16 order 2", 65536, 1024, 4096, 16, 2, 20)


if __name__ == "__main__":
    main()
