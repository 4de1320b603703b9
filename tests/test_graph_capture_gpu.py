"""The library enqueues kernels on the caller's stream and nothing else (no allocation, no synchronisation, no
memset nodes), so a step can be captured into a HIP graph and replayed.  Every replay is checked against the eager
result, with eager work and synchronisations between the replays."""
import numpy as np
import pytest

from paper_2411_00999_amd import workloads
import parity_util as pu

pytestmark = pytest.mark.gpu


def _eager_noise(torch):
    a = torch.randn(1 << 20, device="cuda")
    return float((a * a).sum())


def test_layernorm_step_replays_from_a_graph():
    import torch
    from paper_2411_00999_amd import binding
    B, T, D, n_layers = 8, 256, 768, 4
    layers = []
    for l in range(n_layers):
        inp = workloads.make_inputs(2, l, B=B, T=T, D=D)
        f32 = dict(dtype=torch.float32, device="cuda")
        layers.append(dict(x=pu.to_device(inp.x, "bf16"), dy=pu.to_device(inp.dy, "bf16"),
                           gamma=pu.to_device(inp.gamma, "bf16"), dx=torch.empty((B, T, D), dtype=torch.bfloat16, device="cuda"),
                           dg=torch.empty(D, **f32), db=torch.empty(D, **f32),
                           ws=binding.alloc_workspace(B, T, D, binding.BF16)))
    pe = torch.zeros((2 * n_layers, B), dtype=torch.float32, device="cuda")
    big = torch.zeros(2 * n_layers, dtype=torch.float32, device="cuda")
    gns = torch.zeros(5, dtype=torch.float32, device="cuda")
    all_ws = [L["ws"] for L in layers]

    def step():
        for l, L in enumerate(layers):
            binding.ln_bwd_pegn(L["x"], L["dy"], L["gamma"], workloads.EPS, dx=L["dx"], dgamma=L["dg"], dbeta=L["db"],
                                pe_gamma_sq=pe[2 * l], pe_beta_sq=pe[2 * l + 1], big_sq=big[2 * l:2 * l + 2],
                                workspace=L["ws"], deferred=True)
        binding.reduce_deferred(all_ws, B, T, D, binding.BF16)
        binding.gns_estimate(pe, big, float(B), out=gns)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (pe, big, gns)] + [L[k].clone() for L in layers for k in ("dx", "dg", "db")]

    step()
    want = snapshot()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                       # warm-up on the capture stream
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for replay in range(3):
        for t in (pe, big, gns):
            t.fill_(-1.0)
        for L in layers:
            L["dx"].zero_(); L["dg"].fill_(7.0); L["db"].fill_(7.0)
        _eager_noise(torch)
        graph.replay()
        got = snapshot()
        assert all(torch.equal(a, b) for a, b in zip(got, want)), f"replay {replay}"


def test_linear_and_embedding_replay_from_a_graph():
    import torch
    from paper_2411_00999_amd import binding
    lib = binding.load()
    B, T, K, L, V = 3, 130, 264, 136, 500
    x, g = workloads.make_linear_inputs(5, B, T, K, L, "bf16")
    xd, gd = pu.to_device(x, "bf16"), pu.to_device(g, "bf16")
    ids, ge = workloads.make_embedding_inputs(5, B, T, K, V, "bf16")
    idd, ged = torch.from_numpy(ids).cuda(), pu.to_device(ge, "bf16")
    f32 = dict(dtype=torch.float32, device="cuda")
    w1, s1, b1 = torch.empty((K, L), **f32), torch.empty(B, **f32), torch.empty(1, **f32)
    w2, s2, b2 = torch.empty((V, K), **f32), torch.empty(B, **f32), torch.empty(1, **f32)
    ws1 = torch.empty(max(256, lib.linear_pegn_workspace_bytes(B, T, K, L, binding.BF16)), dtype=torch.uint8, device="cuda")
    ws2 = torch.empty(lib.embedding_pegn_workspace_bytes(B, T, K, V), dtype=torch.uint8, device="cuda")

    def step():
        binding.linear_pegn(xd, gd, w=w1, s=s1, big_sq=b1, workspace=ws1)
        binding.embedding_pegn(idd, ged, V, w=w2, s=s2, big_sq=b2, workspace=ws2)   # forks its fill and joins it

    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in (w1, s1, b1, w2, s2, b2)]
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for replay in range(3):
        for t in (w1, s1, b1, w2, s2, b2):
            t.fill_(3.0)
        _eager_noise(torch)
        graph.replay()
        torch.cuda.synchronize()
        got = [w1, s1, b1, w2, s2, b2]
        assert all(torch.equal(a, b) for a, b in zip(got, want)), f"replay {replay}"
