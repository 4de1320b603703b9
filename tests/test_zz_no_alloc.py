"""The entry point that allocates nothing (ln_bwd_pegn_static) against ln_bwd_pegn, through the C ABI:
two calls in a row on one GPU, the second with a smaller input, so that whatever the first call left in
the library's fixed scratch is still there when the second runs."""
import numpy as np
import pytest

import oracle
import parity_util as pu
from paper_2411_00999_amd import workloads

pytestmark = pytest.mark.gpu


def _buffers(B, T, D, dtype):
    import torch
    f32 = dict(dtype=torch.float32, device="cuda")
    dx = torch.empty((B, T, D), dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device="cuda")
    return dict(dx=dx, dgamma=torch.empty(D, **f32), dbeta=torch.empty(D, **f32),
                pe_gamma_sq=torch.empty(B, **f32), pe_beta_sq=torch.empty(B, **f32), big_sq=torch.empty(2, **f32))


def _both_ways(inp, saved):
    import torch
    from paper_2411_00999_amd import binding
    x, dy, gamma = (pu.to_device(a, inp.dtype) for a in (inp.x, inp.dy, inp.gamma))
    mean, rstd = binding.ln_fwd_stats(x, inp.eps) if saved else (None, None)
    want = binding.ln_bwd_pegn(x, dy, gamma, inp.eps, mean=mean, rstd=rstd)
    out = _buffers(inp.B, inp.T, inp.D, inp.dtype)
    for t in out.values():
        t.fill_(float("nan"))
    torch.cuda.synchronize()
    got = binding.ln_bwd_pegn_static(x, dy, gamma, inp.eps, mean=mean, rstd=rstd, **out)
    torch.cuda.synchronize()
    return got, want


# first call, then a smaller second call; vector kernels with several chunks per example, one workgroup
# per example (B > 256), the generic kernel (odd D), fp32
SEQUENCES = [
    [(3, 8, 256, 2048), (3, 2, 50, 2048)],
    [(4, 300, 8, 1024), (2, 3, 37, 768)],
    [(5, 2, 64, 8192), (1, 4, 128, 256)],
    [(1, 3, 40, 1001), (1, 1, 7, 257)],
]


@pytest.mark.parametrize("seq", SEQUENCES, ids=lambda s: "->".join("x".join(map(str, c[1:])) for c in s))
@pytest.mark.parametrize("saved", [False, True])
def test_static_scratch_call_matches_workspace_call(seq, saved):
    import torch
    for cfg, B, T, D in seq:
        inp = workloads.make_inputs(cfg, B=B, T=T, D=D)
        got, want = _both_ways(inp, saved)
        for name, g, w in zip(("dx", "dgamma", "dbeta", "pe_gamma_sq", "pe_beta_sq", "big_sq"), got, want):
            assert torch.equal(g, w), f"{name} differs from ln_bwd_pegn at B={B} T={T} D={D}"
        # and, like every other path, against the oracle
        ref = oracle.ln_bwd_pegn(inp.x, inp.dy, inp.gamma, inp.eps, want_pe=False)
        res = dict(dx=pu.to_host64(got[0]), dgamma=pu.to_host64(got[1]), dbeta=pu.to_host64(got[2]),
                   s_gamma=pu.to_host64(got[3]), s_beta=pu.to_host64(got[4]), big_sq=pu.to_host64(got[5]))
        pu.compare_with_oracle(inp, res, ref)


def test_full_size_benchmark_shapes_fit_and_match():
    """Workload 4 (B=512: the largest per-example table) then workload 2, full size, device-drawn data."""
    import torch
    from paper_2411_00999_amd import binding
    torch.manual_seed(7)
    for B, T, D in ((512, 64, 1024), (8, 1024, 768)):
        x = torch.randn((B, T, D), device="cuda").to(torch.bfloat16)
        dy = (torch.randn((B, T, D), device="cuda") * 1e-3).to(torch.bfloat16)
        gamma = (1 + 0.05 * torch.randn(D, device="cuda")).to(torch.bfloat16)
        want = binding.ln_bwd_pegn(x, dy, gamma, 1e-5)
        out = _buffers(B, T, D, "bf16")
        got = binding.ln_bwd_pegn_static(x, dy, gamma, 1e-5, **out)
        torch.cuda.synchronize()
        for g, w in zip(got, want):
            assert torch.equal(g, w)


def test_largest_benchmark_shape_fits_the_fixed_scratch():
    """B=8 T=4096 D=8192 bf16 needs 33 MiB of chunk sums; inputs drawn on the device, results compared bit for bit
    with the workspace call (the oracle comparison of this shape is test_full_size_workloads)."""
    import torch
    from paper_2411_00999_amd import binding
    B, T, D = 8, 4096, 8192
    gen = torch.Generator(device="cuda").manual_seed(5)
    x = torch.randn((B, T, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    dy = torch.randn((B, T, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    gamma = (1.0 + 0.1 * torch.randn(D, generator=gen, device="cuda")).to(torch.bfloat16)
    want = binding.ln_bwd_pegn(x, dy, gamma, 1e-5)
    out = _buffers(B, T, D, "bf16")
    got = binding.ln_bwd_pegn_static(x, dy, gamma, 1e-5, **out)
    torch.cuda.synchronize()
    for name, g, w in zip(("dx", "dgamma", "dbeta", "pe_gamma_sq", "pe_beta_sq", "big_sq"), got, want):
        assert torch.equal(g, w), name
    assert torch.isfinite(got[3]).all() and float(got[5][0]) > 0.0


def test_static_scratch_call_replays_from_a_graph():
    """What the entry point is for: a caller under HIP graph capture, which cannot allocate.  The first call on
    the device is made outside the capture (it looks the scratch address up); the captured step then allocates
    nothing, and every replay gives the eager results bit for bit, with eager work in between."""
    import torch
    from paper_2411_00999_amd import binding
    B, T, D = 4, 96, 2048
    inp = workloads.make_inputs(3, B=B, T=T, D=D)
    x, dy, gamma = (pu.to_device(a, inp.dtype) for a in (inp.x, inp.dy, inp.gamma))
    out = _buffers(B, T, D, "bf16")
    pe = torch.empty((2, B), dtype=torch.float32, device="cuda")
    gns = torch.empty(5, dtype=torch.float32, device="cuda")

    def step():
        binding.ln_bwd_pegn_static(x, dy, gamma, inp.eps, out["dx"], out["dgamma"], out["dbeta"], pe[0], pe[1],
                                   out["big_sq"])
        binding.gns_estimate(pe, out["big_sq"], float(B), out=gns)

    step()
    torch.cuda.synchronize()
    tensors = [out[k] for k in ("dx", "dgamma", "dbeta", "big_sq")] + [pe, gns]
    want = [t.clone() for t in tensors]
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for replay in range(3):
        for t in tensors:
            t.fill_(-1.0)
        a = torch.randn(1 << 20, device="cuda")
        float((a * a).sum())                     # eager work and a synchronisation between the replays
        graph.replay()
        torch.cuda.synchronize()
        assert all(torch.equal(g, w) for g, w in zip(tensors, want)), f"replay {replay}"


def test_shape_beyond_the_fixed_scratch_is_refused():
    """Host validation only: nothing is launched, the fake pointers are never dereferenced."""
    import ctypes
    from paper_2411_00999_amd import binding
    lib = binding.load()
    B, T, D = 4096, 8, 8192
    assert lib.lnpegn_workspace_bytes(B, T, D, binding.BF16) > binding.STATIC_SCRATCH_BYTES
    P = ctypes.c_void_p
    p = [P(0x10000 * (i + 1)) for i in range(9)]
    rc = lib.ln_bwd_pegn_static(p[0], p[1], p[2], None, None, p[3], p[4], p[5], p[6], p[7], p[8], B, T, D,
                                binding.BF16, binding.BF16, 1e-5, None)
    assert rc == 3      # LNPEGN_EWORKSPACE
    assert lib.ln_bwd_pegn_static(p[0], p[1], p[2], None, None, p[3], p[4], p[5], p[6], p[7], p[8], 0, T, D,
                                  binding.BF16, binding.BF16, 1e-5, None) == 1
