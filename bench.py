#!/usr/bin/env python3
"""Benchmark of the Monarch Mixer hot path on one MI355X.

A step is one pass of the whole fused path (pad -> Monarch DFT -> (.) k_f -> inverse Monarch DFT
-> truncate, gates fused) over one batch of the configuration the metric is quoted on:
the causal Monarch-FFT long convolution with B=8, H=768, n=1024 zero-padded to 2048 = 64 x 32,
bf16 in / fp32 accumulate.  Inputs are seeded synthetic tensors already resident in HBM; the
step rotates through enough distinct buffer sets (> 512 MB) that the 256 MB Infinity Cache
cannot serve them.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
# HBM bytes per launch of the timed kernel from rocprofv3 FETCH_SIZE / WRITE_SIZE, each scaled by what
# the same counter reads for a plain copy (0.5 and 1.0): profiles/conv2048_bf16_c2_hbm_traffic.txt
MEASURED_TRAFFIC_BYTES = int((19388.5 / 0.5 + 12288.0 / 1.0) * 1024)
WORKLOAD = "c2_conv"


def _make_set(torch, cfg, seed, canonical=None):
    """One buffer set on the device.  Set 0 is the seeded numpy workload (also checked against
    the oracle); the others are fresh draws of the same distributions made on the device."""
    B, H, n = cfg["B"], cfg["H"], cfg["n"]
    if canonical is not None:
        return {k: (None if v is None else torch.from_numpy(v).cuda().to(torch.bfloat16)) for k, v in canonical.items()}
    g = torch.Generator(device="cuda").manual_seed(1000 + seed)
    u = torch.randn((B, H, n), device="cuda", generator=g)
    t = torch.arange(n, device="cuda", dtype=torch.float32)
    k = torch.randn((H, n), device="cuda", generator=g) * torch.exp(-0.01 * t)[None]
    W1 = torch.randn((H, H), device="cuda", generator=g) / H ** 0.5
    W2 = torch.randn((H, H), device="cuda", generator=g) / H ** 0.5
    g_in = torch.matmul(W1.t()[None], u)
    g_out = torch.matmul(W2.t()[None], u)
    return {"u": u.bfloat16(), "k": k.bfloat16(), "g_in": g_in.bfloat16(), "g_out": g_out.bfloat16()}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (rows are independent, so more GPUs "
              "would just split the batch); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2310_12109_amd import binding, costmodel, workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = workloads.CONFIGS[WORKLOAD]
    B, H, n, factors = cfg["B"], cfg["H"], cfg["n"], cfg["factors"]

    canonical = workloads.conv_inputs(B, H, n, cfg["seed"], gates=cfg["gates"], bf16=True)
    bytes_per_step = costmodel.conv_algorithmic_bytes(B, H, n, n, dtype_bytes=2, gates=2)
    nsets = max(2, int(np.ceil(512e6 / bytes_per_step)) + 1)
    sets = [_make_set(torch, cfg, 0, canonical)] + [_make_set(torch, cfg, s) for s in range(1, nsets)]
    outs = [torch.empty_like(s["u"]) for s in sets]
    ws_bytes = binding.monarch_causal_conv_workspace_bytes(B, H, n, n, factors, binding.BF16)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")

    def step(i):
        s = sets[i % nsets]
        binding.monarch_causal_conv(s["u"], s["k"], s["g_in"], s["g_out"], factors, causal=True, ws=ws, out=outs[i % nsets])

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    # One pass over all buffer sets is captured into a HIP graph (the step is a single ~15 us
    # kernel: launching it from Python call by call would time the interpreter, not the GPU).
    # The timed region replays it and runs the remainder eagerly: exactly `steps` steps.
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for i in range(nsets):
            step(i)
    graph.replay()
    torch.cuda.synchronize()
    start, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    start.record()
    for _ in range(args.steps // nsets):
        graph.replay()
    for i in range(args.steps % nsets):
        step(i)
    end.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ev_ms = start.elapsed_time(end)
    ms_per_step = ev_ms / args.steps
    value = B * n * H / (ms_per_step * 1e-3)

    achieved_gbs = bytes_per_step / (ms_per_step * 1e-3) / 1e9
    flops = costmodel.conv_executed_flops(B, H, factors)

    out = {
        "metric": "M2 mixer tokens/s (B*N*H)", "value": value, "unit": "elements/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "causal Monarch-FFT conv B=8 H=768 n=1024 nfft=2048=64x32, gates fused, bf16 in / fp32 acc",
                   "B": B, "H": H, "n": n, "nfft": int(np.prod(factors)), "factors": list(factors),
                   "buffer_sets": nsets, "launch": "hip graph of %d steps, replayed" % nsets, "sequence_tokens_per_s": B * n / (ms_per_step * 1e-3)},
        "roofline": {"bound": "hbm", "achieved": achieved_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved_gbs / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC_BYTES,
                     "kernel": "conv2048_bf16_kernel", "algorithmic_bytes_per_launch": bytes_per_step,
                     "executed_tflops": flops / (ms_per_step * 1e-3) / 1e12},
        "host_wall_ms_per_step": wall_ms / args.steps,
    }

    # parity of the timed configuration against the oracle, and the oracle's own speed
    if not args.no_cpu_baseline:
        import oracle
        reps = []
        want = None
        for _ in range(3):
            t1 = time.perf_counter()
            want = oracle.causal_conv(canonical["u"], canonical["k"], canonical["g_in"], canonical["g_out"], nfft=2048)
            reps.append(time.perf_counter() - t1)
        cpu_s = sorted(reps)[1]
        step(0)
        torch.cuda.synchronize()
        got = outs[0].float().cpu().numpy().astype(np.float64)
        out["rel_l2_vs_oracle"] = float(np.linalg.norm(got - want) / np.linalg.norm(want))
        out["cpu_baseline"] = {"value": B * n * H / cpu_s, "unit": "elements/s", "cores": oracle.num_threads(),
                               "kind": "oracle", "sample": "the full batch (8 x 768 rows of 1024), direct O(n^2) sum in "
                               "fp64, median of 3 runs (%.2f s each)" % cpu_s}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
