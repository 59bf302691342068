"""The fused convolution launched from a replayed HIP graph gives the eager result every time."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL_BF16, announce, dev, host, rel_l2
from paper_2310_12109_amd import workloads

pytestmark = pytest.mark.gpu


def test_graph_replays_match_eager():
    from paper_2310_12109_amd import binding
    announce("conv graph replay")
    w = workloads.conv_inputs(4, 16, 1024, seed=3, gates="normal", bf16=True)
    t = {k: dev(v, True) for k, v in w.items()}
    eager = binding.monarch_causal_conv(t["u"], t["k"], t["g_in"], t["g_out"], (64, 32))
    torch.cuda.synchronize()
    want = eager.clone()
    out = torch.empty_like(eager)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        binding.monarch_causal_conv(t["u"], t["k"], t["g_in"], t["g_out"], (64, 32), out=out)   # warm up on this stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        binding.monarch_causal_conv(t["u"], t["k"], t["g_in"], t["g_out"], (64, 32), out=out)
    for rep in range(4):
        out.zero_()
        # eager work and a synchronisation between the replays
        other = binding.monarch_causal_conv(t["g_in"], t["k"], None, None, (64, 32))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want), f"replay {rep} differs from the eager result"
        assert other.shape == want.shape
    # and the replayed result is the right one, not merely the repeated one: the oracle's direct sum
    ref = oracle.causal_conv(w["u"], w["k"], w["g_in"], w["g_out"], nfft=2048)
    assert rel_l2(host(out), ref) <= TOL_BF16


def test_graph_replays_of_the_matmul_gradients_match_eager():
    # dR / dL are cleared by a fill kernel inside the call (no memset node) and summed with atomics: every replay
    # must start from zero again and agree with the eager result to rounding
    from paper_2310_12109_amd import binding
    announce("matmul backward graph replay")
    w = workloads.monarch_matmul_inputs(batch=3000, b=16, seed=4)
    x, R, L = dev(w["x"]), dev(w["R"]), dev(w["L"])
    dy = dev(np.random.default_rng(5).standard_normal((3000, 256)).astype(np.float32))
    _, wantR, wantL = binding.monarch_matmul_backward(x, R, L, dy, need_dx=False)
    torch.cuda.synchronize()
    outs = {}
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        outs["dx"], outs["dR"], outs["dL"] = binding.monarch_matmul_backward(x, R, L, dy)
    for rep in range(3):
        binding.monarch_matmul(x, R, L)   # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in ((outs["dR"], wantR), (outs["dL"], wantL)):
            err = float((got - want).norm() / want.norm())
            assert err <= 1e-5, f"replay {rep}: {err}"


def test_graph_replays_of_the_layer_and_the_blocky_convolution_match_eager():
    # two-kernel entry points (layer: workspace between the kernels; blocky: prepared state) captured and replayed
    from paper_2310_12109_amd import binding
    announce("layer + blocky conv graph replay")
    w = workloads.m2_layer_inputs(3, 16, 16, seed=6)
    d = {k: dev(v) for k, v in w.items()}
    seq, dim = [d[k] for k in ("R1", "L1", "R2", "L2")], [d[k] for k in ("R3", "L3", "R4", "L4")]
    ws = torch.empty(binding.monarch_m2_layer_workspace_bytes(3, 256, 256, binding.F32), dtype=torch.uint8, device="cuda")
    want_layer = binding.monarch_m2_layer(d["x"], seq, d["n_kernel"], dim, d["d_kernel"], d["gamma"], d["beta"], ws=ws).clone()
    wb = workloads.blocky_inputs(3, 20, 128, 16, seed=7)
    state = binding.monarch_blocky_prepare(dev(wb["Lt"]), dev(wb["Rt"]), dev(wb["k"]), mask=True)
    u, gi, go = dev(wb["u"]), dev(wb["g_in"]), dev(wb["g_out"])
    want_conv = binding.monarch_blocky_conv(u, gi, go, state, 16).clone()
    torch.cuda.synchronize()
    out_layer, out_conv = torch.empty_like(want_layer), torch.empty_like(want_conv)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        binding.monarch_m2_layer(d["x"], seq, d["n_kernel"], dim, d["d_kernel"], d["gamma"], d["beta"], ws=ws, out=out_layer)
        binding.monarch_blocky_conv(u, gi, go, state, 16, out=out_conv)
    for rep in range(3):
        out_layer.zero_(); out_conv.zero_(); ws.zero_()
        binding.monarch_mixer(u.new_zeros(1, 4, 256), u.new_zeros(4, 256), None, None, *seq)   # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_layer, want_layer), f"layer: replay {rep} differs from the eager result"
        assert torch.equal(out_conv, want_conv), f"blocky conv: replay {rep} differs from the eager result"
