#!/usr/bin/env python3
"""Benchmark of the Monarch Mixer hot path on one MI355X: the one measurement program of this repository.

Headline (`value`, `ms_per_step`, `roofline`): a step is one pass of the whole fused path
(pad -> Monarch DFT -> (.) k_f -> inverse Monarch DFT -> truncate, gates fused) over one batch of the
configuration the metric is quoted on: the causal Monarch-FFT long convolution with B=8, H=768, n=1024
zero-padded to 2048 = 64 x 32, bf16 in / fp32 accumulate.  `configs` carries the same measurement for every
other named configuration (Monarch matmul at batch 2^20, the fp32 convolution, the M2-BERT-shaped convolution
and MLP, the 128 x 128 and 64^3 long convolutions, the 16-block MLP).

How a case is timed: inputs are seeded synthetic tensors already resident in HBM; a case rotates through
enough distinct buffer sets (> 512 MB) that the 256 MB Infinity Cache cannot serve them; the launches of one
pass over the sets are captured into a HIP graph; a timed region is exactly `steps` steps (replays of that graph
plus one of a shorter graph for the remainder), bracketed by HIP events on the stream the kernels run on; the region is repeated until
at least 50 ms have been timed and the median region is reported.  Prints ONE JSON line.

  python bench.py                       headline + every configuration + oracle baseline
  python bench.py --config c4_conv      one configuration only (what the rocprofv3 commands in profiles/ run)
  python bench.py --copy-calibration 256   plain copies of 256 MiB (calibrates FETCH_SIZE / WRITE_SIZE)
  python bench.py --summarize-profile DIR [--kernel NAME]   medians of a rocprofv3 output folder (no GPU needed)
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_TFLOPS = 2500.0      # dense bf16 matrix peak, published
MFMA_F32_TFLOPS = 157.3        # fp32 matrix peak, published
HEADLINE = "c2_conv_bf16"
MIN_TIMED_MS = 50.0


def traffic_from_profile(name):
    """HBM bytes per launch of a case's dominant kernel as the counter run measured them: the line
    `TRAFFIC <case> <bytes>` of profiles/hbm_traffic.txt (written from rocprofv3 FETCH_SIZE / WRITE_SIZE runs of
    this program, each scaled by what the counter reads for a plain copy).  None when no such line exists."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        m = re.match(r"\s*TRAFFIC\s+(\S+)\s+(\d+)", line)
        if m and m.group(1) == name:
            return int(m.group(2))
    return None


class Case:
    """One configuration: buffer sets on the device, the call, the cost model, the parity sample."""
    name = ""
    workload = ""
    dtype = "bf16"
    kernel = ""

    def build(self, torch, binding, workloads):      # -> list of zero-argument callables, one per buffer set
        raise NotImplementedError

    def elements(self):                              # the "(B*N*H)" unit of the metric
        raise NotImplementedError

    def algorithmic_bytes(self):
        raise NotImplementedError

    def executed_flops(self):
        return 0.0

    bound = "hbm"
    mfma_peak = MFMA_BF16_TFLOPS

    def parity(self, np, torch, oracle):             # -> (rel_l2, description) of buffer set 0 against the oracle
        return None, ""

    def roofline(self, ms):
        t = ms * 1e-3
        gbs = self.algorithmic_bytes() / t / 1e9
        tf = self.executed_flops() / t / 1e12
        r = {"bound": self.bound, "kernel": self.kernel, "algorithmic_bytes_per_step": self.algorithmic_bytes(),
             "executed_flops_per_step": self.executed_flops(), "hbm_gbs": gbs, "executed_tflops": tf,
             "traffic": traffic_from_profile(self.name)}
        if self.bound == "hbm":
            r.update(achieved=gbs, peak=HBM_PEAK_GBS, unit="GB/s", frac=gbs / HBM_PEAK_GBS)
        else:
            r.update(achieved=tf, peak=self.mfma_peak, unit="TFLOP/s", frac=tf / self.mfma_peak)
        return r


def _nsets(bytes_per_set, cap=24):
    return max(2, min(cap, int(512e6 // max(bytes_per_set, 1)) + 2))


def _rel(np, got, want):
    return float(np.linalg.norm(np.asarray(got, dtype=np.float64) - want) / np.linalg.norm(want))


class ConvCase(Case):
    def __init__(self, name, cfg_key, bf16, kernel, bound="hbm", mfma_peak=MFMA_BF16_TFLOPS, launches=1):
        self.name, self.cfg_key, self.bf16, self.kernel, self.bound, self.mfma_peak = name, cfg_key, bf16, kernel, bound, mfma_peak
        self.dtype = "bf16" if bf16 else "f32"
        self.launches = launches

    def build(self, torch, binding, workloads):
        from paper_2310_12109_amd import costmodel
        self.costmodel = costmodel
        c = workloads.CONFIGS[self.cfg_key]
        self.B, self.H, self.n, self.factors, self.gates = c["B"], c["H"], c["n"], tuple(c["factors"]), c["gates"]
        B, H, n = self.B, self.H, self.n
        nfft = 1
        for f in self.factors:
            nfft *= f
        self.nfft = nfft
        self.workload = ("causal Monarch-FFT conv B=%d H=%d n=%d nfft=%d=%s, gates fused, %s" %
                         (B, H, n, nfft, "x".join(map(str, self.factors)), "bf16 in / fp32 acc" if self.bf16 else "fp32"))
        tdt = torch.bfloat16 if self.bf16 else torch.float32
        self.canonical = workloads.conv_inputs(B, H, n, c["seed"], gates=self.gates, bf16=self.bf16)
        first = {k: (None if v is None else torch.from_numpy(v).cuda().to(tdt)) for k, v in self.canonical.items()}
        nsets = _nsets(self.algorithmic_bytes())
        self.sets = [first]
        t = torch.arange(n, device="cuda", dtype=torch.float32)
        for s in range(1, nsets):
            g = torch.Generator(device="cuda").manual_seed(1000 + s)
            u = torch.randn((B, H, n), device="cuda", generator=g)
            k = torch.randn((H, n), device="cuda", generator=g) * torch.exp(-0.01 * t)[None]
            if self.gates == "projected":
                W1 = torch.randn((H, H), device="cuda", generator=g) / H ** 0.5
                W2 = torch.randn((H, H), device="cuda", generator=g) / H ** 0.5
                g_in, g_out = torch.matmul(W1.t()[None], u), torch.matmul(W2.t()[None], u)
            else:
                g_in = torch.randn((B, H, n), device="cuda", generator=g)
                g_out = torch.randn((B, H, n), device="cuda", generator=g)
            self.sets.append({"u": u.to(tdt), "k": k.to(tdt), "g_in": g_in.to(tdt), "g_out": g_out.to(tdt)})
            del u, k, g_in, g_out
        self.outs = [torch.empty_like(s["u"]) for s in self.sets]
        ws_bytes = binding.monarch_causal_conv_workspace_bytes(B, H, n, n, self.factors, binding.BF16 if self.bf16 else binding.F32)
        ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")

        def call(i):
            s = self.sets[i]
            return lambda: binding.monarch_causal_conv(s["u"], s["k"], s["g_in"], s["g_out"], self.factors, causal=True, ws=ws, out=self.outs[i])
        return [call(i) for i in range(nsets)]

    def elements(self):
        return self.B * self.n * self.H

    def algorithmic_bytes(self):
        es = 2 if self.bf16 else 4
        return (2 + 2) * self.B * self.H * self.n * es + self.H * self.n * es

    def executed_flops(self):
        return self.costmodel.conv_executed_flops(self.B, self.H, self.factors)

    def parity(self, np, torch, oracle):
        w = self.canonical
        got = self.outs[0].float().cpu().numpy().astype(np.float64)
        rows_total = self.B * self.H
        if rows_total * self.n * self.n <= 2e10:       # the whole tensor by the direct sum
            want = oracle.causal_conv(w["u"], w["k"], w["g_in"], w["g_out"], nfft=self.nfft)
            return _rel(np, got, want), "every output, direct O(n^2) sum in fp64"
        rng = np.random.default_rng(0)
        npts = 4096
        rows = rng.integers(0, rows_total, size=npts)
        ts = rng.integers(0, self.n, size=npts)
        ts[:4] = (0, 1, self.n // 2, self.n - 1)
        want = oracle.causal_conv_points(w["u"], w["k"], w["g_in"], w["g_out"], rows, ts, nfft=self.nfft)
        return _rel(np, got.reshape(rows_total, self.n)[rows, ts], want), "%d seeded outputs, direct O(n) sums in fp64" % npts


class MatmulCase(Case):
    name = "c1_matmul_f32_batch_2p20"
    dtype = "f32"
    kernel = "monarch_b16_kernel<float>"
    batch = 1 << 20

    def build(self, torch, binding, workloads):
        self.workload = "order-2 Monarch matmul N=256 (16 blocks of 16x16), fp32, batch 2^20 (config 1's kernel at steady state)"
        w = workloads.monarch_matmul_inputs(batch=4096, b=16, seed=0)
        self.canonical = w
        R, L = torch.from_numpy(w["R"]).cuda(), torch.from_numpy(w["L"]).cuda()
        g = torch.Generator(device="cuda").manual_seed(7)
        self.x = torch.randn((self.batch, 256), device="cuda", generator=g)
        self.x[:4096] = torch.from_numpy(w["x"]).cuda()
        self.y = torch.empty_like(self.x)
        self.x2 = torch.randn((self.batch, 256), device="cuda", generator=g)
        self.y2 = torch.empty_like(self.x2)
        return [lambda: binding.monarch_matmul(self.x, R, L, out=self.y), lambda: binding.monarch_matmul(self.x2, R, L, out=self.y2)]

    def elements(self):
        return self.batch * 256

    def algorithmic_bytes(self):
        return (2 * self.batch * 256 + 2 * 16 * 256) * 4

    def executed_flops(self):
        return self.batch * 4.0 * 256 * 16

    def parity(self, np, torch, oracle):
        w = self.canonical
        got = self.y[:4096].cpu().numpy()
        return _rel(np, got, oracle.matmul(w["x"], w["R"], w["L"])), "the first 4096 vectors against the dense 256x256 product in fp64"


class MlpCase(Case):
    def __init__(self, name, cfg_key, order, kernel, bound):
        self.name, self.cfg_key, self.order, self.kernel, self.bound = name, cfg_key, order, kernel, bound

    def build(self, torch, binding, workloads):
        from paper_2310_12109_amd import costmodel
        self.costmodel = costmodel
        c = workloads.CONFIGS[self.cfg_key]
        self.tokens, self.d, self.dh, self.nb = c["tokens"], c["d"], c["d_hidden"], c["nb"]
        self.workload = "Monarch MLP order %d, %d tokens, %d -> %d -> %d, %d blocks, GELU, bf16" % (
            self.order, self.tokens, self.d, self.dh, self.d, self.nb)
        w = workloads.mlp_inputs(self.tokens, self.d, self.dh, self.nb, self.order, c["seed"], bf16=True)
        self.canonical = w
        bf = lambda a: None if a is None else torch.from_numpy(a).cuda().to(torch.bfloat16)
        wt = {k: bf(w[k]) for k in ("W1_R", "W1_L", "b1", "W2_R", "W2_L", "b2")}
        nsets = _nsets(self.algorithmic_bytes())
        g = torch.Generator(device="cuda").manual_seed(11)
        self.xs = [bf(w["x"])] + [torch.randn((self.tokens, self.d), device="cuda", generator=g).to(torch.bfloat16) for _ in range(nsets - 1)]
        self.ys = [torch.empty_like(x) for x in self.xs]
        ws_bytes = binding.monarch_mlp_workspace_bytes(self.tokens, self.d, self.dh, self.nb, self.order, 0, 0, binding.BF16)
        ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")

        def call(i):
            return lambda: binding.monarch_mlp(self.xs[i], wt["W1_R"], wt["W1_L"], wt["b1"], wt["W2_R"], wt["W2_L"], wt["b2"],
                                               self.nb, self.order, 2, self.dh, ws=ws, out=self.ys[i])
        return [call(i) for i in range(nsets)]

    def elements(self):
        return self.tokens * self.d

    def algorithmic_bytes(self):
        return self.costmodel.mlp_algorithmic_bytes(self.tokens, self.d, self.dh, self.nb, self.order)

    def executed_flops(self):
        return self.costmodel.mlp_flops(self.tokens, self.d, self.dh, self.nb, self.order)

    def parity(self, np, torch, oracle):
        w = self.canonical
        rows = np.sort(np.random.default_rng(0).choice(self.tokens, size=128, replace=False))
        rows[0], rows[-1] = 0, self.tokens - 1
        want = oracle.mlp(w["x"][rows], w["W1_R"], w["W1_L"], w["b1"], w["W2_R"], w["W2_L"], w["b2"], nb=self.nb, order=self.order, act=2)
        got = self.ys[0].float().cpu().numpy()[rows]
        return _rel(np, got, want), "128 seeded tokens against the dense-materialised MLP in fp64"


class RandomCase(Case):
    """A case of the widening rows (learned mixer, gradients, order 3, the basic layer, the blocky convolution, the
    plain transforms): random tensors of the stated shapes, timed like every other case; their parity with the
    oracle is the business of tests/, so no sample is checked here.  `make(torch, binding, rnd)` returns a function
    that builds one buffer set and returns its call."""
    def __init__(self, name, workload, dtype, kernel, nbytes, flops, elements, make, bound="hbm", mfma_peak=MFMA_F32_TFLOPS):
        self.name, self.workload, self.dtype, self.kernel = name, workload, dtype, kernel
        self._bytes, self._flops, self._elements, self._make = nbytes, flops, elements, make
        self.bound, self.mfma_peak = bound, mfma_peak

    def build(self, torch, binding, workloads):
        def rnd(*shape, dt=torch.float32, scale=1.0):
            return (torch.randn(*shape, device="cuda") * scale).to(dt)
        one = self._make(torch, binding, workloads, rnd)
        return [one() for _ in range(_nsets(self._bytes))]

    def elements(self):
        return self._elements

    def algorithmic_bytes(self):
        return self._bytes

    def executed_flops(self):
        return self._flops


def widening_cases():
    """Cases that only run when named with --config (what the rocprofv3 commands of profiles/ use)."""
    cases = []

    def add(*a, **k):
        cases.append(RandomCase(*a, **k))

    def tdt(torch, name):
        return torch.bfloat16 if name == "bf16" else torch.float32

    for batch in (64, 1 << 20):
        for dn in ("f32", "bf16"):
            es = 4 if dn == "f32" else 2

            def mk_fwd(torch, binding, workloads, rnd, batch=batch, dn=dn):
                dt = tdt(torch, dn)
                R, L = rnd(16, 16, 16, dt=dt, scale=.25), rnd(16, 16, 16, dt=dt, scale=.25)

                def one():
                    x = rnd(batch, 256, dt=dt)
                    y = torch.empty_like(x)
                    return lambda: binding.monarch_matmul(x, R, L, out=y)
                return one

            def mk_bwd(torch, binding, workloads, rnd, batch=batch, dn=dn):
                dt = tdt(torch, dn)
                R, L = rnd(16, 16, 16, dt=dt, scale=.25), rnd(16, 16, 16, dt=dt, scale=.25)

                def one():
                    x, dy = rnd(batch, 256, dt=dt), rnd(batch, 256, dt=dt)
                    return lambda: binding.monarch_matmul_backward(x, R, L, dy)
                return one
            add("c1_matmul_%s_batch_%d" % (dn, batch), "order-2 Monarch matmul N=256, %s, batch %d" % (dn, batch), dn,
                "monarch_b16_kernel", (2 * batch * 256 + 2 * 4096) * es, batch * 4.0 * 256 * 16, batch * 256, mk_fwd)
            add("c1_backward_%s_batch_%d" % (dn, batch), "gradients of the order-2 Monarch matmul N=256, %s, batch %d" % (dn, batch), dn,
                "matmul_backward_b16_kernel", 3 * batch * 256 * es + 2 * 4096 * (es + 4), batch * 10.0 * 256 * 16, batch * 256, mk_bwd)

    # square products and the mixer with blocks of 32 and 64 (N = 1024, 4096): in place on LDS tiles, fp32 MFMA
    for b, B in ((32, 128), (64, 32)):
        for dn in ("f32", "bf16"):
            es = 4 if dn == "f32" else 2
            N, rows = b * b, B * 768

            def mk_mm_b(torch, binding, workloads, rnd, b=b, N=N, rows=rows, dn=dn):
                dt = tdt(torch, dn)
                R, L = rnd(b, b, b, dt=dt, scale=b ** -0.5), rnd(b, b, b, dt=dt, scale=b ** -0.5)

                def one():
                    x = rnd(rows, N, dt=dt)
                    y = torch.empty_like(x)
                    return lambda: binding.monarch_matmul(x, R, L, out=y)
                return one

            def mk_mixer_b(torch, binding, workloads, rnd, b=b, N=N, B=B, dn=dn):
                dt = tdt(torch, dn)
                K = rnd(768, N, dt=dt)
                f = [rnd(b, b, b, dt=dt, scale=b ** -0.5) for _ in range(4)]

                def one():
                    u, gi, go = (rnd(B, 768, N, dt=dt) for _ in range(3))
                    y = torch.empty_like(u)
                    return lambda: binding.monarch_mixer(u, K, gi, go, *f, out=y)
                return one
            add("matmul_%s_b%d_batch_%d" % (dn, b, rows), "order-2 Monarch matmul N=%d (%d blocks of %dx%d), %s, batch %d" % (N, b, b, b, dn, rows),
                dn, "inpl::matmul_kernel<%d>" % b, (2 * rows * N + 2 * b ** 3) * es, rows * 4.0 * N * b, rows * N, mk_mm_b)

            def mk_mm_bwd_b(torch, binding, workloads, rnd, b=b, N=N, rows=rows, dn=dn):
                dt = tdt(torch, dn)
                R, L = rnd(b, b, b, dt=dt, scale=b ** -0.5), rnd(b, b, b, dt=dt, scale=b ** -0.5)

                def one():
                    x, dy = rnd(rows, N, dt=dt), rnd(rows, N, dt=dt)
                    return lambda: binding.monarch_matmul_backward(x, R, L, dy)
                return one
            add("matmul_backward_%s_b%d_batch_%d" % (dn, b, rows), "gradients of the order-2 Monarch matmul N=%d, %s, batch %d" % (N, dn, rows),
                dn, "inpl::backward_dx_dl_kernel + backward_dr_kernel" if b == 32 else "inpl::backward64_dx_kernel + 2 x backward64_factor_kernel",
                3 * rows * N * es + 2 * b ** 3 * (es + 4), rows * 10.0 * N * b, rows * N, mk_mm_bwd_b)
            add("mixer_%s_b%d_B%d" % (dn, b, B), "learned-Monarch sequence mixer N=%d, B=%d H=768, %s" % (N, B, dn), dn,
                "inpl::mixer_kernel<%d>" % b, (4 * rows * N + 768 * N + 4 * b ** 3) * es, rows * 8.0 * N * b, rows * N, mk_mixer_b)

    for B in (8, 1024):
        for dn in ("f32", "bf16"):
            es = 4 if dn == "f32" else 2
            rows = B * 768

            def mk_mixer(torch, binding, workloads, rnd, B=B, dn=dn):
                dt = tdt(torch, dn)
                K = rnd(768, 256, dt=dt)
                f = [rnd(16, 16, 16, dt=dt, scale=.25) for _ in range(4)]

                def one():
                    u, gi, go = (rnd(B, 768, 256, dt=dt) for _ in range(3))
                    y = torch.empty_like(u)
                    return lambda: binding.monarch_mixer(u, K, gi, go, *f, out=y)
                return one

            def mk_blocky(torch, binding, workloads, rnd, B=B, dn=dn):
                dt = tdt(torch, dn)
                w = workloads.blocky_inputs(1, 768, 128, 16, seed=0)
                state = binding.monarch_blocky_prepare(*(torch.from_numpy(w[k]).cuda() for k in ("Lt", "Rt", "k")), mask=True)

                def one():
                    u, gi, go = (rnd(B, 768, 128, dt=dt) for _ in range(3))
                    y = torch.empty_like(u)
                    return lambda: binding.monarch_blocky_conv(u, gi, go, state, 16, out=y)
                return one
            add("mixer_%s_B%d" % (dn, B), "learned-Monarch sequence mixer N=256, B=%d H=768, %s" % (B, dn), dn, "mixer_b16_kernel",
                (4 * rows * 256 + 768 * 256 + 4 * 4096) * es, rows * 8.0 * 256 * 16, rows * 256, mk_mixer)
            add("blocky_conv_%s_B%d" % (dn, B), "polynomial-parameterised Monarch causal conv N=256 n=128, B=%d H=768, %s" % (B, dn), dn,
                "blocky16::conv_b16_kernel", 4 * rows * 128 * es + 768 * 256 * 8 + 4 * 4096 * 8, rows / 16 * 704 * 2048.0, rows * 128,
                mk_blocky, bound="mfma")

    for dn in ("f32", "bf16"):   # the same convolution at N = 1024 (blocks of 32), n = 512: in place on LDS tiles
        es = 4 if dn == "f32" else 2

        def mk_blocky32(torch, binding, workloads, rnd, dn=dn):
            dt = tdt(torch, dn)
            w = workloads.blocky_inputs(1, 768, 512, 32, seed=0)
            state = binding.monarch_blocky_prepare(*(torch.from_numpy(w[k]).cuda() for k in ("Lt", "Rt", "k")), mask=True)

            def one():
                u, gi, go = (rnd(64, 768, 512, dt=dt) for _ in range(3))
                y = torch.empty_like(u)
                return lambda: binding.monarch_blocky_conv(u, gi, go, state, 32, out=y)
            return one
        rows32 = 64 * 768
        # executed MFMAs per tile of 16 rows: 512 (real input) + 2048 + 2048 + 512 (real part, half of the rows), 2048 FLOP each
        add("blocky_conv_%s_b32_B64" % dn, "polynomial-parameterised Monarch causal conv N=1024 n=512, B=64 H=768, %s" % dn, dn,
            "inpl::blocky_kernel<32>", 4 * rows32 * 512 * es + 768 * 1024 * 8 + 4 * 32768 * 8, rows32 / 16 * 5120 * 2048.0, rows32 * 512,
            mk_blocky32, bound="mfma")

    for B, dn in ((8, "f32"), (256, "f32"), (256, "bf16")):
        es = 4 if dn == "f32" else 2

        def mk_mixb(torch, binding, workloads, rnd, B=B, dn=dn):
            dt = tdt(torch, dn)
            K = rnd(768, 256, dt=dt)
            f = [rnd(16, 16, 16, dt=dt, scale=.25) for _ in range(4)]
            ws = torch.empty(binding.raw().monarch_mixer_backward_workspace_bytes(B, 768, 16, binding.F32 if dn == "f32" else binding.BF16),
                             dtype=torch.uint8, device="cuda")

            def one():
                u, gi, go, dy = (rnd(B, 768, 256, dt=dt) for _ in range(4))
                return lambda: binding.monarch_mixer_backward(u, K, gi, go, *f, dy, ws=ws)
            return one
        add("mixer_backward_%s_B%d" % (dn, B), "gradients of the learned mixer N=256, B=%d H=768, %s" % (B, dn), dn, "composition (9 launches)",
            7 * B * 768 * 256 * es, B * 768 * 28.0 * 256 * 16, B * 768 * 256, mk_mixb)

    for B, dn in ((32, "f32"), (2048, "f32"), (2048, "bf16")):
        es = 4 if dn == "f32" else 2

        def mk_layer(torch, binding, workloads, rnd, B=B, dn=dn):
            dt = tdt(torch, dn)
            w = workloads.m2_layer_inputs(1, 16, 16, seed=0)
            par = {k: torch.from_numpy(v).cuda().to(dt) for k, v in w.items() if k != "x"}
            seq, dim = [par[k] for k in ("R1", "L1", "R2", "L2")], [par[k] for k in ("R3", "L3", "R4", "L4")]
            ws = torch.empty(binding.monarch_m2_layer_workspace_bytes(B, 256, 256, binding.F32 if dn == "f32" else binding.BF16),
                             dtype=torch.uint8, device="cuda")

            def one():
                x = rnd(B, 256, 256, dt=dt)
                y = torch.empty_like(x)
                return lambda: binding.monarch_m2_layer(x, seq, par["n_kernel"], dim, par["d_kernel"], par["gamma"], par["beta"], ws=ws, out=y)
            return one
        add("m2_layer_%s_B%d" % (dn, B), "basic M2 layer n=d=256, B=%d, %s" % (B, dn), dn, "mixer_b16_kernel (2 launches)",
            (4 * B * 65536 + 2 * 65536) * es, B * 512 * 16.0 * 256 * 16, B * 65536, mk_layer)

    for dn in ("f32", "bf16"):   # the layer at n = d = 1024: both mixers in place on the matrix cores
        es = 4 if dn == "f32" else 2

        def mk_layer32(torch, binding, workloads, rnd, dn=dn):
            dt = tdt(torch, dn)
            w = workloads.m2_layer_inputs(1, 32, 32, seed=0)
            par = {k: torch.from_numpy(v).cuda().to(dt) for k, v in w.items() if k != "x"}
            seq, dim = [par[k] for k in ("R1", "L1", "R2", "L2")], [par[k] for k in ("R3", "L3", "R4", "L4")]
            ws = torch.empty(binding.monarch_m2_layer_workspace_bytes(64, 1024, 1024, binding.F32 if dn == "f32" else binding.BF16),
                             dtype=torch.uint8, device="cuda")

            def one():
                x = rnd(64, 1024, 1024, dt=dt)
                y = torch.empty_like(x)
                return lambda: binding.monarch_m2_layer(x, seq, par["n_kernel"], dim, par["d_kernel"], par["gamma"], par["beta"], ws=ws, out=y)
            return one
        add("m2_layer_%s_b32_B64" % dn, "basic M2 layer n=d=1024, B=64, %s" % dn, dn, "inpl::mixer_kernel<32> (2 launches)",
            (4 * 64 * 1048576 + 2 * 1048576) * es, 64 * 2048 * 16.0 * 1024 * 32, 64 * 1048576, mk_layer32)

    for b, batch in ((8, 16384), (16, 4096), (16, 65536)):
        N = b ** 3

        def mk_mm3(torch, binding, workloads, rnd, b=b, batch=batch, N=N, backward=False):
            f = [rnd(b * b, b, b, scale=b ** -0.5) for _ in range(3)]

            def one():
                x = rnd(batch, N)
                if backward:
                    dy = rnd(batch, N)
                    return lambda: binding.monarch_matmul3_backward(x, *f, dy)
                y = torch.empty_like(x)
                return lambda: binding.monarch_matmul3(x, *f, out=y)
            return one
        add("matmul3_f32_b%d_batch_%d" % (b, batch), "general order-3 Monarch product N=%d, fp32, batch %d" % (N, batch), "f32",
            "mm3b16::forward_kernel" if b == 16 else "mm3::forward_kernel", 2 * batch * N * 4 + 3 * N * b * 4, batch * 6.0 * N * b, batch * N, mk_mm3)
        if True:
            add("matmul3_backward_f32_b%d_batch_%d" % (b, batch), "gradients of the order-3 Monarch product N=%d, fp32, batch %d" % (N, batch), "f32",
                "mm3b16::backward_kernel (3 launches)" if b == 16 else "mm3::backward_kernel", 3 * batch * N * 4 + 6 * N * b * 4, batch * 16.0 * N * b, batch * N,
                lambda torch, binding, workloads, rnd, f=mk_mm3: f(torch, binding, workloads, rnd, backward=True))

    # the general order-p product (shape-generic LDS-tile kernels) at N = 4096 = 8^4 and 4^6
    for b, p, batch in ((8, 4, 16384), (4, 6, 16384)):
        N = b ** p

        def mk_mmp(torch, binding, workloads, rnd, b=b, p=p, batch=batch, N=N, backward=False):
            f = rnd(p, N // b, b, b, scale=b ** -0.5)

            def one():
                x = rnd(batch, N)
                if backward:
                    dy = rnd(batch, N)
                    return lambda: binding.monarch_matmulp_backward(x, f, dy)
                y = torch.empty_like(x)
                return lambda: binding.monarch_matmulp(x, f, out=y)
            return one
        add("matmulp_f32_b%d_p%d_batch_%d" % (b, p, batch), "general order-%d Monarch product N=%d, fp32, batch %d" % (p, N, batch), "f32",
            "mmp::forward_kernel", 2 * batch * N * 4 + p * N * b * 4, batch * 2.0 * p * N * b, batch * N, mk_mmp)
        add("matmulp_backward_f32_b%d_p%d_batch_%d" % (b, p, batch), "gradients of the order-%d Monarch product N=%d, fp32, batch %d" % (p, N, batch),
            "f32", "mmp::backward_kernel", 3 * batch * N * 4 + 2 * p * N * b * 4, batch * (6.0 * p - 2.0) * N * b, batch * N,
            lambda torch, binding, workloads, rnd, f=mk_mmp: f(torch, binding, workloads, rnd, backward=True))

    # the gated-convolution layer at the shape of config 2 (B = 8, n = 1024, d = 768): four dense projections (rocBLAS),
    # the short convolutions and the fused long convolution
    for dn in ("bf16", "f32"):
        es = 4 if dn == "f32" else 2
        B, n, d = 8, 1024, 768

        def mk_hy(torch, binding, workloads, rnd, dn=dn, B=B, n=n, d=d):
            dt = tdt(torch, dn)
            W_in, W_out = rnd(3 * d, d, dt=dt, scale=d ** -0.5), rnd(d, d, dt=dt, scale=d ** -0.5)
            b_in, b_out = rnd(3 * d, dt=dt, scale=.1), rnd(d, dt=dt, scale=.1)
            k_short, k_long = rnd(3 * d, 3, dt=dt, scale=.5), rnd(d, n, dt=dt, scale=.1)
            ws = torch.empty(max(16, binding.monarch_hyena_layer_workspace_bytes(B, n, d, n, (64, 32), dt)), dtype=torch.uint8, device="cuda")

            def one():
                u = rnd(B, n, d, dt=dt)
                y = torch.empty_like(u)
                return lambda: binding.monarch_hyena_layer(u, W_in, b_in, k_short, k_long, W_out, b_out, (64, 32), ws=ws, out=y)
            return one
        add("hyena_layer_%s_B8_n1024_d768" % dn, "gated-convolution layer (projections, short convs, gated long conv) B=8 n=1024 d=768, %s" % dn,
            dn, "rocBLAS GEMMs + short_conv_kernel + conv2048 kernel", (2 * B * n * d + 4 * d * d + d * n) * es,
            8.0 * B * n * d * d, B * n * d, mk_hy, bound="mfma", mfma_peak=MFMA_BF16_TFLOPS if dn == "bf16" else MFMA_F32_TFLOPS)

    # the same layer with heads of 16 features (the head dimension of the paper's causal models): 256 long convolutions
    # per head and batch entry
    from paper_2310_12109_amd import costmodel
    for dn in ("bf16", "f32"):
        es = 4 if dn == "f32" else 2
        B, n, d, dh = 8, 1024, 768, 16

        def mk_hyh(torch, binding, workloads, rnd, dn=dn, B=B, n=n, d=d, dh=dh):
            dt = tdt(torch, dn)
            W_in, W_out = rnd(3 * d, d, dt=dt, scale=d ** -0.5), rnd(d, d, dt=dt, scale=d ** -0.5)
            b_in, b_out = rnd(3 * d, dt=dt, scale=.1), rnd(d, dt=dt, scale=.1)
            k_short, k_long = rnd(3 * d, 3, dt=dt, scale=.5), rnd(d // dh, n, dt=dt, scale=.1)
            ws = torch.empty(max(16, binding.monarch_hyena_heads_layer_workspace_bytes(B, n, d, n, (64, 32), dh, dt)), dtype=torch.uint8,
                             device="cuda")

            def one():
                u = rnd(B, n, d, dt=dt)
                y = torch.empty_like(u)
                return lambda: binding.monarch_hyena_heads_layer(u, W_in, b_in, k_short, k_long, W_out, b_out, (64, 32), dh, ws=ws, out=y)
            return one
        add("hyena_heads_layer_%s_B8_n1024_d768_dh16" % dn,
            "gated-convolution layer with heads of 16 features B=8 n=1024 d=768, %s" % dn, dn,
            "rocBLAS GEMMs + short_conv_kernel + conv2048 kernel (outer products on its loads) + heads_sum_kernel" if dn == "bf16"
            else "rocBLAS GEMMs + short_conv_kernel + heads_outer_kernel + conv2048 kernel + heads_sum_kernel",
            (2 * B * n * d + 4 * d * d + (d // dh) * n) * es, 8.0 * B * n * d * d + costmodel.conv_executed_flops(B * dh * dh, d // dh, (64, 32)),
            B * n * d, mk_hyh, bound="mfma",
            mfma_peak=MFMA_BF16_TFLOPS if dn == "bf16" else MFMA_F32_TFLOPS)

    for rows, factors in ((6144, (64, 32)), (1536, (128, 128))):
        N = factors[0] * factors[1]
        for inverse in (False, True):
            def mk_fft(torch, binding, workloads, rnd, rows=rows, factors=factors, N=N, inverse=inverse):
                def one():
                    if inverse:
                        X = torch.randn((rows, N, 2), dtype=torch.float32, device="cuda")
                        x = torch.empty((rows, N), dtype=torch.bfloat16, device="cuda")
                        return lambda: binding.monarch_ifft(X, factors, True, dtype=torch.bfloat16, out=x)
                    x = rnd(rows, N, dt=torch.bfloat16)
                    X = torch.empty((rows, N, 2), dtype=torch.float32, device="cuda")
                    return lambda: binding.monarch_fft(x, factors, True, out=X)
                return one
            add("%s_bf16_%dx%d" % ("ifft" if inverse else "fft", rows, N), "Monarch %s, %d real bf16 rows of %d = %dx%d, fp32 spectrum" % (
                "inverse DFT" if inverse else "DFT", rows, N, factors[0], factors[1]), "bf16", "fft2_lds_kernel", rows * N * 10, 0.0, rows * N, mk_fft)
    return cases


def all_cases():
    return [
        ConvCase("c2_conv_bf16", "c2_conv", True, "conv2048_kernel<bf16>", "hbm"),
        MatmulCase(),
        ConvCase("c2_conv_f32", "c2_conv", False, "conv2048_f32_kernel", "mfma", MFMA_F32_TFLOPS),
        ConvCase("c3a_conv_bf16", "c3a_conv", True, "conv256_bf16_kernel", "hbm"),
        MlpCase("c3b_mlp_order1", "c3b_mlp", 1, "mlp_order1_split_kernel", "mfma"),
        MlpCase("c3b_mlp_order2", "c3b_mlp", 2, "factor_kernel + mlp_order1 + factor_kernel", "mfma"),
        ConvCase("c4_conv_bf16", "c4_conv", True, "conv16k_bf16_kernel", "mfma"),
        ConvCase("c5a_conv_bf16", "c5a_conv", True, "fft_pass_rows_in_kernel x 2 + conv3_middle_kernel<64,64> + fft_pass_rows_out_kernel (4 launches)", "mfma"),
        MlpCase("c5b_mlp_order1", "c5b_mlp", 1, "mlp_order1_resident_kernel", "hbm"),
        MlpCase("c5b_mlp_order2", "c5b_mlp", 2, "factor_resident_kernel + mlp_order1_resident_kernel + factor_resident_kernel", "hbm"),
    ]


def time_case(torch, calls, steps, warmup):
    """Median time of a region of exactly `steps` steps, in ms per step; regions repeat until >= MIN_TIMED_MS."""
    nsets = len(calls)
    for i in range(max(warmup, 1)):
        calls[i % nsets]()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for c in calls:
            c()
    graph.replay()
    rest = None                      # the steps of a region that do not fill a whole pass: a second graph
    if steps % nsets:
        rest = torch.cuda.CUDAGraph()
        with torch.cuda.graph(rest):
            for c in calls[:steps % nsets]:
                c()
        rest.replay()
    torch.cuda.synchronize()
    regions, total_ms, host_ms = [], 0.0, 0.0
    while (total_ms < MIN_TIMED_MS or len(regions) < 3) and len(regions) < 2000:
        start, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        start.record()
        for _ in range(steps // nsets):
            graph.replay()
        if rest is not None:
            rest.replay()
        end.record()
        torch.cuda.synchronize()
        host_ms += (time.perf_counter() - t0) * 1e3
        regions.append(start.elapsed_time(end))
        total_ms += regions[-1]
    regions.sort()
    med = regions[len(regions) // 2]
    return {"ms_per_step": med / steps, "regions": len(regions), "region_ms_min": regions[0], "region_ms_max": regions[-1],
            "host_wall_ms_per_step": host_ms / (len(regions) * steps), "buffer_sets": nsets}


def run_case(torch, np, binding, workloads, oracle, case, steps, warmup, check):
    calls = case.build(torch, binding, workloads)
    t = time_case(torch, calls, steps, warmup)
    ms = t["ms_per_step"]
    rec = {"name": case.name, "workload": case.workload, "dtype": case.dtype, "steps": steps, "ms_per_step": ms,
           "value": case.elements() / (ms * 1e-3), "unit": "elements/s", "roofline": case.roofline(ms)}
    rec.update({k: t[k] for k in ("regions", "region_ms_min", "region_ms_max", "host_wall_ms_per_step", "buffer_sets")})
    if check:
        calls[0]()
        torch.cuda.synchronize()
        rel, how = case.parity(np, torch, oracle)
        rec["rel_l2_vs_oracle"] = rel
        rec["parity_sample"] = how
    return rec


def copy_calibration(mib):
    """Plain device-to-device copies of a known size: what FETCH_SIZE / WRITE_SIZE read for known traffic, and (under
    a kernel trace) what a kernel that only moves bytes reaches at that size.  The copies rotate over source /
    destination pairs of more than 512 MB in total, like the timed cases."""
    import torch
    n = mib * (1 << 20)
    pairs = _nsets(2 * n, cap=16)
    bufs = [(torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 255), torch.empty(n, dtype=torch.uint8, device="cuda"))
            for _ in range(pairs)]
    copies = max(8, 4 * pairs)
    for i in range(copies):
        src, dst = bufs[i % pairs]
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"copy_calibration_mib": mib, "copies": copies, "buffer_pairs": pairs}))


def summarize_profile(directory, kernel_filter):
    """Prints what the text files under profiles/ quote from a rocprofv3 output folder: per kernel whose name
    contains `kernel_filter`, the median and mean per dispatch of every collected counter
    (*_counter_collection.csv) and the rows of the kernel statistics (*_kernel_stats.csv)."""
    import collections
    import csv
    import glob
    for path in sorted(glob.glob(os.path.join(directory, "**", "*_counter_collection.csv"), recursive=True)):
        acc = collections.defaultdict(lambda: collections.defaultdict(list))
        with open(path, newline="") as f:
            for row in csv.DictReader(f):
                if kernel_filter in row["Kernel_Name"]:
                    acc[row["Kernel_Name"]][row["Counter_Name"]].append(float(row["Counter_Value"]))
        for name, counters in acc.items():
            print("%s\n  %s" % (path, name[:120]))
            for cname, v in sorted(counters.items()):
                v.sort()
                print("    %-32s dispatches %5d  median %16.1f  mean %16.1f" % (cname, len(v), v[len(v) // 2], sum(v) / len(v)))
    for path in sorted(glob.glob(os.path.join(directory, "**", "*_kernel_stats.csv"), recursive=True)):
        with open(path, newline="") as f:
            for row in csv.DictReader(f):
                if kernel_filter in row["Name"]:
                    print("%s\n  %s\n    calls %s  total ns %s  average ns %s  min %s  max %s" % (
                        path, row["Name"][:120], row["Calls"], row["TotalDurationNs"], row["AverageNs"], row["MinNs"], row["MaxNs"]))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3500, help="steps of the headline case per timed region")
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", action="append", help="run only these cases (names as in the `configs` list); the first is the headline of the line")
    ap.add_argument("--no-extra-configs", action="store_true", help="headline only")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle legs (parity samples and the oracle timing)")
    ap.add_argument("--copy-calibration", type=int, metavar="MIB", help="only run plain copies of this size (counter calibration)")
    ap.add_argument("--summarize-profile", metavar="DIR", help="only print counter / kernel-trace summaries of a rocprofv3 output folder")
    ap.add_argument("--kernel", default="monarch", help="with --summarize-profile: substring a kernel name must contain")
    args = ap.parse_args()
    if args.summarize_profile:
        summarize_profile(args.summarize_profile, args.kernel)
        return
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (rows are independent, so more GPUs "
              "would just split the batch); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.copy_calibration:
        copy_calibration(args.copy_calibration)
        return

    import numpy as np
    import torch

    from paper_2310_12109_amd import binding, workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    oracle = None
    if not args.no_cpu_baseline:
        import oracle

    cases = {c.name: c for c in all_cases()}
    default_names = list(cases)
    cases.update({c.name: c for c in widening_cases()})
    if args.config:
        unknown = [n for n in args.config if n not in cases]
        if unknown:
            sys.exit("bench.py: unknown case(s) %s; known: %s" % (unknown, ", ".join(cases)))
        order = args.config
    else:
        order = [HEADLINE] + ([] if args.no_extra_configs else [n for n in default_names if n != HEADLINE])

    head_case = cases[order[0]]
    head = run_case(torch, np, binding, workloads, oracle, head_case, args.steps, args.warmup, oracle is not None)
    out = {
        "metric": "M2 mixer tokens/s (B*N*H)", "value": head["value"], "unit": "elements/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": head_case.dtype, "data": "synthetic",
        "config": {"workload": head["workload"], "case": head["name"], "buffer_sets": head["buffer_sets"],
                   "launch": "hip graph of one pass over the buffer sets, replayed; %d regions of %d steps, median" % (head["regions"], args.steps),
                   "region_ms_min": head["region_ms_min"], "region_ms_max": head["region_ms_max"]},
        "roofline": head["roofline"],
        "host_wall_ms_per_step": head["host_wall_ms_per_step"],
    }
    if hasattr(head_case, "B"):
        out["config"]["sequence_tokens_per_s"] = head_case.B * head_case.n / (head["ms_per_step"] * 1e-3)
    if "rel_l2_vs_oracle" in head:
        out["rel_l2_vs_oracle"] = head["rel_l2_vs_oracle"]

    # the oracle's own speed on the headline workload (a reported baseline, not a target)
    if oracle is not None and isinstance(head_case, ConvCase):
        w = head_case.canonical
        rows_total = head_case.B * head_case.H
        sample_rows = max(1, min(rows_total, int(2e11 // (head_case.n * head_case.n))))    # bounds the CPU work
        b_rows = max(1, sample_rows // head_case.H)
        h_rows = min(head_case.H, sample_rows)          # a long sequence: only some channels of one batch entry
        sub = {k: (None if w[k] is None else w[k][:b_rows, :h_rows]) for k in ("u", "g_in", "g_out")}
        reps = []
        for _ in range(3):
            t1 = time.perf_counter()
            oracle.causal_conv(sub["u"], w["k"][:h_rows], sub["g_in"], sub["g_out"], nfft=head_case.nfft)
            reps.append(time.perf_counter() - t1)
        cpu_s = sorted(reps)[1]
        out["cpu_baseline"] = {"value": b_rows * h_rows * head_case.n / cpu_s, "unit": "elements/s", "cores": oracle.num_threads(),
                               "kind": "oracle", "sample": "%d of %d batch entries (%d rows of %d), direct O(n^2) sum in fp64, "
                               "median of 3 runs (%.2f s each)" % (b_rows, head_case.B, b_rows * h_rows, head_case.n, cpu_s)}
    del head_case
    cases[order[0]] = None
    torch.cuda.empty_cache()

    extra = []
    for name in order[1:]:
        case = cases[name]
        try:
            extra.append(run_case(torch, np, binding, workloads, oracle, case, _steps_for(case), min(args.warmup, 5), oracle is not None))
        finally:
            cases[name] = None
            del case
            torch.cuda.empty_cache()
    if extra:
        out["configs"] = extra
    print(json.dumps(out))


def _steps_for(case):
    """Steps per timed region of a non-headline case: short kernels get more so that a region is not a handful
    of microseconds; every region is still repeated until 50 ms have been timed."""
    if isinstance(case, ConvCase) and case.cfg_key == "c3a_conv":
        return 440
    if isinstance(case, MlpCase) and case.cfg_key == "c3b_mlp":
        return 240
    if isinstance(case, ConvCase) and case.cfg_key == "c2_conv":
        return 100
    if isinstance(case, RandomCase) and case.algorithmic_bytes() < 64e6:
        return 200
    return 12


if __name__ == "__main__":
    main()
