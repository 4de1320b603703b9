"""GPU parity tests: the HIP path, called through the C ABI, against the fp64 CPU oracle on the
same seeded inputs, element by element.  Run with `pytest -m gpu` on an MI355X."""
import numpy as np
import pytest

import oracle
from paper_2411_00999_amd import workloads
import parity_util as pu

pytestmark = pytest.mark.gpu


def _oracle(inp, want_dx=True):
    return oracle.ln_bwd_pegn(inp.x, inp.dy, inp.gamma, inp.eps, want_dx=want_dx, want_pe=False)


def _gns_both(res, ref, B):
    """End-to-end estimate: GPU norms through the GPU estimator vs oracle norms through the oracle."""
    import torch
    from paper_2411_00999_amd import binding
    d = res["_dev"]
    out = binding.gns_estimate(torch.stack([d["sg"], d["sb"]]), d["big"], float(B))
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    want = oracle.gns_estimate(np.stack([ref["s_gamma"], ref["s_beta"]]), ref["big_sq"], float(B))
    return got, want


def _check_gns(got, want, B):
    keys = ("g_small_sq", "g_big_sq", "G2", "S", "B_simple")
    w = np.array([want[k] for k in keys])
    # norms and S are well conditioned
    np.testing.assert_allclose(got[:2], w[:2], rtol=pu.TOL_SUMS)
    np.testing.assert_allclose(got[3], w[3], rtol=pu.TOL_GNS)
    # G2 (Eq. 4) is a difference of nearly equal numbers when the true gradient is ~0: the
    # synthetic dy is zero-mean.  kappa is the amplification of a relative error in the norms.
    kappa = pu.gns_condition(B, want["g_big_sq"], want["g_small_sq"])
    eps_norm = 2.0 ** -23       # the norms are handed over as fp32
    rtol = max(pu.TOL_GNS, 4 * kappa * eps_norm)
    assert got[2] == pytest.approx(w[2], rel=rtol), ("G2", kappa)
    assert got[4] == pytest.approx(w[4], rel=2 * rtol), ("B_simple", kappa)


# ------------------------------------------------------------------ workload 1, full size
@pytest.mark.parametrize("saved", [False, True])
@pytest.mark.parametrize("signal", [0.0, 1e-2])
def test_workload1_fp32_pegn_and_gns(saved, signal):
    inp = workloads.make_inputs(1, signal=signal)
    ref = _oracle(inp)
    res = pu.run_gpu(inp, saved_stats=saved)
    pu.compare_with_oracle(inp, res, ref)
    got, want = _gns_both(res, ref, inp.B)
    _check_gns(got, want, inp.B)
    if signal > 0:      # well conditioned: the plain 1e-4 bar holds on every output
        keys = ("g_small_sq", "g_big_sq", "G2", "S", "B_simple")
        np.testing.assert_allclose(got, [want[k] for k in keys], rtol=pu.TOL_GNS)
        assert want["B_simple"] > 0
    if saved:
        m, r = oracle.ln_stats(inp.x, inp.eps)
        pu.check_close("mean", res["mean"], m, pu.TOL_F32)
        np.testing.assert_allclose(res["rstd"], r, rtol=pu.TOL_F32)


def test_workload1_plain_matches_oracle_and_fused():
    inp = workloads.make_inputs(1)
    ref = _oracle(inp)
    plain = pu.run_gpu(inp, pegn=False)
    pu.compare_with_oracle(inp, plain, ref, pegn=False)
    fused = pu.run_gpu(inp)
    np.testing.assert_array_equal(plain["dx"], fused["dx"])     # same row arithmetic


# ------------------------------------------------------------------ reduced shapes of 2..5
REDUCED = [
    # (workload, B, T, D): several chunks, several column tiles, ragged row counts
    (2, 3, 37, 768),
    (2, 2, 130, 576),
    (2, 5, 19, 960),
    (3, 2, 150, 2048),
    (3, 3, 41, 4096),
    (4, 16, 8, 1024),
    (4, 70, 3, 1024),
    (5, 2, 33, 8192),
    (5, 1, 70, 6144),
]


@pytest.mark.parametrize("cfg,B,T,D", REDUCED)
@pytest.mark.parametrize("saved", [False, True])
def test_reduced_workloads_bf16(cfg, B, T, D, saved):
    inp = workloads.make_inputs(cfg, B=B, T=T, D=D)
    ref = _oracle(inp)
    res = pu.run_gpu(inp, saved_stats=saved)
    pu.compare_with_oracle(inp, res, ref)
    if B > 1:
        got, want = _gns_both(res, ref, B)
        _check_gns(got, want, B)
    plain = pu.run_gpu(inp, saved_stats=saved, pegn=False)
    pu.compare_with_oracle(inp, plain, ref, pegn=False)


@pytest.mark.parametrize("B,T,D,dtype", [
    (2, 9, 1, "f32"), (3, 5, 5, "f32"), (2, 11, 257, "f32"), (2, 7, 258, "f32"), (2, 6, 1028, "f32"),
    (2, 9, 1, "bf16"), (3, 5, 7, "bf16"), (2, 11, 257, "bf16"), (2, 5, 1001, "bf16"), (1, 4, 9000, "bf16"),
    (2, 5, 12288, "bf16"), (2, 3, 2048, "f32"), (2, 3, 8192, "f32"), (2, 9, 64, "f32"), (2, 9, 8, "bf16"),
])
def test_any_D_is_correct(B, T, D, dtype):
    """Generic kernel (odd D, D above the tuned range) and the small/large ends of the tuned ones."""
    inp = workloads.make_inputs(1, B=B, T=T, D=D, dtype=dtype)
    ref = _oracle(inp)
    for saved in (False, True):
        res = pu.run_gpu(inp, saved_stats=saved)
        pu.compare_with_oracle(inp, res, ref)


@pytest.mark.parametrize("B,T,D,dtype", [
    (3, 70, 1280, "bf16"),      # two waves per row, lanes left over: four row groups
    (2, 90, 1536, "bf16"),
    (2, 41, 1600, "bf16"),
    (3, 50, 2560, "bf16"),      # three waves per row (run-time wave count), two row groups, padded
    (2, 64, 3072, "bf16"),      # ... full rows
    (2, 33, 5120, "bf16"),      # five waves
    (2, 40, 6144, "bf16"),      # six waves
    (2, 21, 7168, "bf16"),      # seven waves
    (3, 37, 1280, "f32"),       # fp32: two waves of three vectors, padded
    (2, 50, 1536, "f32"),
    (2, 33, 3072, "f32"),       # three waves of four vectors
    (2, 18, 5120, "f32"),       # beyond eight waves of four vectors: five to eight vectors per lane
])
@pytest.mark.parametrize("saved", [False, True])
def test_row_widths_between_the_powers_of_two(B, T, D, dtype, saved):
    """Every launch shape that the row widths between the benchmark's choose."""
    inp = workloads.make_inputs(3 if dtype == "bf16" else 1, B=B, T=T, D=D, dtype=dtype)
    ref = _oracle(inp)
    res = pu.run_gpu(inp, saved_stats=saved)
    pu.compare_with_oracle(inp, res, ref)
    plain = pu.run_gpu(inp, saved_stats=saved, pegn=False)
    pu.compare_with_oracle(inp, plain, ref, pegn=False)


@pytest.mark.parametrize("B,T,D,dtype", [(2, 33, 12288, "bf16"), (2, 17, 16384, "bf16"), (3, 9, 10240, "bf16"),
                                         (2, 9, 12288, "f32"), (1, 5, 16384, "f32"), (2, 7, 9216, "f32"),
                                         (2, 6, 14336, "f32")])
@pytest.mark.parametrize("saved", [False, True])
def test_rows_wider_than_8192(B, T, D, dtype, saved):
    """Rows beyond eight waves of 16 elements per lane: 24 or 32 elements per lane, still the vector kernels."""
    inp = workloads.make_inputs(5 if dtype == "bf16" else 1, B=B, T=T, D=D, dtype=dtype)
    ref = _oracle(inp)
    res = pu.run_gpu(inp, saved_stats=saved)
    pu.compare_with_oracle(inp, res, ref)
    plain = pu.run_gpu(inp, saved_stats=saved, pegn=False)
    pu.compare_with_oracle(inp, plain, ref, pegn=False)


def test_gamma_fp32_with_bf16_activations():
    inp = workloads.make_inputs(2, B=2, T=40, D=768)
    ref = _oracle(inp)
    res = pu.run_gpu(inp, gamma_f32=True)
    pu.compare_with_oracle(inp, res, ref)


# ------------------------------------------------------------------ edge cases
def test_T1_and_B1():
    for B, T in ((6, 1), (1, 50), (1, 1)):
        inp = workloads.make_inputs(2, B=B, T=T, D=768)
        ref = _oracle(inp)
        res = pu.run_gpu(inp)
        pu.compare_with_oracle(inp, res, ref)
        if B == 1:   # one example: its squared norm IS the squared norm of the batch gradient
            np.testing.assert_allclose(res["s_gamma"][0], res["big_sq"][0], rtol=1e-6)
            np.testing.assert_allclose(res["s_beta"][0], res["big_sq"][1], rtol=1e-6)


def test_constant_row_and_identical_examples():
    inp = workloads.make_inputs(1, B=4, T=16, D=256)
    inp.x[1, 3] = 2.5                                  # sigma^2 = 0 in one row
    inp.x[:] = inp.x[0]
    inp.dy[:] = inp.dy[0]                              # all examples identical
    ref = _oracle(inp)
    res = pu.run_gpu(inp)
    pu.compare_with_oracle(inp, res, ref)
    got, want = _gns_both(res, ref, inp.B)
    big = want["g_big_sq"]
    assert abs(got[3]) <= 1e-5 * big                   # S = 0: no noise
    assert got[2] == pytest.approx(big, rel=1e-5)      # G2 = |G_big|^2


def test_in_place_dx_over_dy():
    inp = workloads.make_inputs(3, B=2, T=30, D=2048)
    ref = _oracle(inp)
    res = pu.run_gpu(inp, in_place=True)
    pu.compare_with_oracle(inp, res, ref)


def test_misaligned_pointers_take_the_generic_kernel():
    import torch
    from paper_2411_00999_amd import binding
    inp = workloads.make_inputs(2, B=2, T=10, D=768)
    ref = _oracle(inp)
    n = inp.B * inp.T * inp.D

    def shifted(a):
        buf = torch.empty(n + 1, dtype=torch.bfloat16, device="cuda")
        view = buf[1:].view(inp.B, inp.T, inp.D)          # 2-byte offset: not 16-byte aligned
        view.copy_(pu.to_device(a, "bf16"))
        return view

    x, dy = shifted(inp.x), shifted(inp.dy)
    gamma = pu.to_device(inp.gamma, "bf16")
    dx, dg, db, sg, sb, big = binding.ln_bwd_pegn(x, dy, gamma, inp.eps)
    torch.cuda.synchronize()
    res = dict(dx=pu.to_host64(dx), dgamma=pu.to_host64(dg), dbeta=pu.to_host64(db),
               s_gamma=pu.to_host64(sg), s_beta=pu.to_host64(sb), big_sq=pu.to_host64(big))
    pu.compare_with_oracle(inp, res, ref)


@pytest.mark.parametrize("B,T,D,dtype", [
    (40, 50, 1024, "bf16"),     # six chunks of consecutive rows per example, the last one short
    (33, 17, 256, "f32"),       # two chunks of 9 and 8 rows
    (200, 130, 768, "bf16"),    # examples cut finer than one round of workgroups: eight chunks of 17, 11 in the last
    (130, 48, 2048, "bf16"),    # too short to cut: a chunk is a whole example, rows of two waves
    (512, 32, 1024, "bf16"),    # a chunk is a whole example, eight rows at a time
    (520, 33, 512, "f32"),      # the same with four rows at a time and a ragged tail
    (300, 100, 1024, "bf16"),   # shapes of the measurements: five blocks of 20 rows per example, three rounds
    (64, 512, 1024, "bf16"),    # eight blocks of 64 rows
    (600, 64, 2048, "bf16"),    # two waves per row, two blocks per example
])
def test_many_short_examples(B, T, D, dtype):
    """More examples than the row kernel has workgroups for: the chunk layouts of that regime."""
    inp = workloads.make_inputs(4 if dtype == "bf16" else 1, B=B, T=T, D=D, dtype=dtype)
    ref = _oracle(inp)
    for saved in (False, True):
        res = pu.run_gpu(inp, saved_stats=saved)
        pu.compare_with_oracle(inp, res, ref)
    got, want = _gns_both(res, ref, B)
    _check_gns(got, want, B)


def test_bitwise_reproducible():
    inp = workloads.make_inputs(3, B=4, T=64, D=2048)
    a = pu.run_gpu(inp)
    for _ in range(10):
        b = pu.run_gpu(inp)
        for k in ("dx", "dgamma", "dbeta", "s_gamma", "s_beta", "big_sq"):
            np.testing.assert_array_equal(a[k], b[k], err_msg=k)


def test_chunk_count_only_changes_summation_order():
    from paper_2411_00999_amd import binding
    inp = workloads.make_inputs(3, B=4, T=96, D=2048)
    ref = _oracle(inp)
    try:
        for chunks in (4, 16, 64, 4096):
            for rows in (1, 2):                         # every C-th row of the example, or a block of rows
                binding.set_tuning(0, chunks)
                binding.set_tuning(1, chunks)
                binding.set_tuning(8, rows)
                res = pu.run_gpu(inp)
                pu.compare_with_oracle(inp, res, ref)
                plain = pu.run_gpu(inp, pegn=False)
                pu.compare_with_oracle(inp, plain, ref, pegn=False)
    finally:
        binding.set_tuning(0, 0)
        binding.set_tuning(1, 0)
        binding.set_tuning(8, 0)


@pytest.mark.parametrize("cfg,B,T,D", [(3, 4, 64, 2048), (2, 3, 37, 768), (4, 300, 4, 1024), (5, 2, 20, 8192),
                                      (1, 2, 9, 257), (4, 40, 50, 1024)])
def test_deferred_reduction_matches_immediate_calls_bitwise(cfg, B, T, D):
    """Several layers of one shape: row passes first, ONE batched reduction afterwards."""
    import torch
    from paper_2411_00999_amd import binding
    n_layers = 5
    dt_code = binding.BF16 if workloads.SHAPES[cfg][3] == "bf16" else binding.F32
    immediate, deferred, wss = [], [], []
    for l in range(n_layers):
        inp = workloads.make_inputs(cfg, layer=l, B=B, T=T, D=D)
        x, dy = pu.to_device(inp.x, inp.dtype), pu.to_device(inp.dy, inp.dtype)
        gamma = pu.to_device(inp.gamma, inp.dtype)
        pegn = l != 2                                   # one plain call mixed in
        if pegn:
            immediate.append(binding.ln_bwd_pegn(x, dy, gamma, inp.eps))
        else:
            immediate.append(binding.ln_bwd(x, dy, gamma, inp.eps))
        ws = binding.alloc_workspace(B, T, D, dt_code)
        wss.append(ws)
        f32 = dict(dtype=torch.float32, device="cuda")
        outs = dict(dgamma=torch.full((D,), float("nan"), **f32), dbeta=torch.full((D,), float("nan"), **f32))
        if pegn:
            outs.update(pe_gamma_sq=torch.full((B,), float("nan"), **f32),
                        pe_beta_sq=torch.full((B,), float("nan"), **f32),
                        big_sq=torch.full((2,), float("nan"), **f32))
            deferred.append(binding.ln_bwd_pegn(x, dy, gamma, inp.eps, workspace=ws, deferred=True, **outs))
        else:
            deferred.append(binding.ln_bwd(x, dy, gamma, inp.eps, workspace=ws, deferred=True, **outs))
    torch.cuda.synchronize()
    assert all(torch.isnan(d[1]).all() for d in deferred)          # nothing but dx written yet
    binding.reduce_deferred(wss, B, T, D, dt_code)
    torch.cuda.synchronize()
    for a, b in zip(immediate, deferred):
        assert len(a) == len(b)
        for u, v in zip(a, b):
            assert torch.equal(u, v)


# ------------------------------------------------------------------ forward, accumulation
def test_deferred_reduction_of_more_layers_than_one_launch_takes():
    """70 layers: lnpegn_reduce_deferred finishes them in two rounds of launches (64 + 6)."""
    import torch
    from paper_2411_00999_amd import binding
    B, T, D, n_layers = 3, 20, 256, 70
    immediate, deferred, wss = [], [], []
    for l in range(n_layers):
        inp = workloads.make_inputs(1, layer=l, B=B, T=T, D=D)
        x, dy, gamma = (pu.to_device(a, inp.dtype) for a in (inp.x, inp.dy, inp.gamma))
        immediate.append(binding.ln_bwd_pegn(x, dy, gamma, inp.eps))
        ws = binding.alloc_workspace(B, T, D, binding.F32)
        wss.append(ws)
        deferred.append(binding.ln_bwd_pegn(x, dy, gamma, inp.eps, workspace=ws, deferred=True))
    binding.reduce_deferred(wss, B, T, D, binding.F32)
    torch.cuda.synchronize()
    for l, (a, b) in enumerate(zip(immediate, deferred)):
        for u, v in zip(a, b):
            assert torch.equal(u, v), l


@pytest.mark.parametrize("cfg,B,T,D", [(1, 4, 128, 256), (2, 3, 37, 768), (3, 2, 50, 2048), (5, 2, 9, 8192),
                                      (1, 2, 7, 257), (2, 2, 5, 1001), (5, 2, 7, 12288), (5, 1, 5, 16384),
                                      (1, 2, 5, 12288), (1, 1, 3, 16384), (5, 1, 3, 20480)])
def test_forward_against_oracle(cfg, B, T, D):
    import torch
    from paper_2411_00999_amd import binding
    inp = workloads.make_inputs(cfg, B=B, T=T, D=D)
    x, gamma, beta = (pu.to_device(a, inp.dtype) for a in (inp.x, inp.gamma, inp.beta))
    y, mean, rstd = binding.ln_fwd(x, gamma, beta, inp.eps)
    torch.cuda.synchronize()
    want = oracle.ln_fwd(inp.x, inp.gamma, inp.beta, inp.eps)
    bf = inp.dtype == "bf16"
    pu.check_close("y", pu.to_host64(y), want, pu.TOL_BF16 if bf else pu.TOL_F32, bf16_output=bf)
    m, r = oracle.ln_stats(inp.x, inp.eps)
    pu.check_close("mean", pu.to_host64(mean), m, pu.TOL_F32, floor_rms=float(np.sqrt(np.mean(inp.x.astype(np.float64) ** 2))))
    np.testing.assert_allclose(pu.to_host64(rstd), r, rtol=pu.TOL_F32)
    y2, none_m, none_r = binding.ln_fwd(x, gamma, beta, inp.eps, want_stats=False)
    torch.cuda.synchronize()
    assert none_m is None and none_r is None and torch.equal(y, y2)
    # the saved statistics feed the backward
    dy = pu.to_device(inp.dy, inp.dtype)
    a = binding.ln_bwd_pegn(x, dy, gamma, inp.eps, mean=mean, rstd=rstd)
    m2, r2 = binding.ln_fwd_stats(x, inp.eps)
    torch.cuda.synchronize()
    assert torch.equal(m2, mean) and torch.equal(r2, rstd)


@pytest.mark.parametrize("cfg,B,T,D,defer", [(3, 4, 40, 2048, False), (2, 3, 21, 768, False),
                                            (4, 300, 2, 1024, False), (3, 4, 40, 2048, True), (1, 2, 9, 257, True),
                                            # one example per micro-batch (Section 5.1's setting), spanning several
                                            # chunks: vector kernel and generic kernel, immediate and deferred
                                            (3, 1, 200, 2048, False), (3, 1, 200, 2048, True),
                                            (1, 1, 50, 257, False), (1, 1, 50, 257, True)])
def test_gradient_accumulation_over_micro_batches(cfg, B, T, D, defer):
    """A micro-batches through LNPEGN_ACCUMULATE == the oracle on the concatenated batch."""
    import torch
    from paper_2411_00999_amd import binding
    A = 3
    inp = workloads.make_inputs(cfg, B=A * B, T=T, D=D)
    ref = oracle.ln_bwd_pegn(inp.x, inp.dy, inp.gamma, inp.eps, want_pe=False)
    dt_code = binding.BF16 if inp.dtype == "bf16" else binding.F32
    f32 = dict(dtype=torch.float32, device="cuda")
    dgamma, dbeta = torch.zeros(D, **f32), torch.zeros(D, **f32)
    pe = torch.zeros((2, A * B), **f32)
    big = torch.zeros(2, **f32)
    gamma = pu.to_device(inp.gamma, inp.dtype)
    flags = binding.PER_EXAMPLE | binding.ACCUMULATE | (binding.DEFER if defer else 0)
    dxs = []
    for a in range(A):
        sl = slice(a * B, (a + 1) * B)
        x, dy = pu.to_device(inp.x[sl], inp.dtype), pu.to_device(inp.dy[sl], inp.dtype)
        ws = binding.alloc_workspace(B, T, D, dt_code)
        dxs.append(binding.ln_bwd_ex(x, dy, gamma, inp.eps, flags, dgamma, dbeta,
                                     pe_gamma_sq=pe[0, sl], pe_beta_sq=pe[1, sl], big_sq=big, workspace=ws))
        if defer:
            binding.reduce_deferred([ws], B, T, D, dt_code)
    torch.cuda.synchronize()
    res = dict(dx=np.concatenate([pu.to_host64(d) for d in dxs]), dgamma=pu.to_host64(dgamma),
               dbeta=pu.to_host64(dbeta), s_gamma=pu.to_host64(pe[0]), s_beta=pu.to_host64(pe[1]),
               big_sq=pu.to_host64(big))
    pu.compare_with_oracle(inp, res, ref)
    out = binding.gns_estimate(pe, big, float(A * B))
    torch.cuda.synchronize()
    want = oracle.gns_estimate(np.stack([ref["s_gamma"], ref["s_beta"]]), ref["big_sq"], float(A * B))
    _check_gns(out.cpu().numpy().astype(np.float64), want, A * B)


# ------------------------------------------------------------------ RMSNorm variant
@pytest.mark.parametrize("cfg,B,T,D", [(1, 4, 128, 256), (2, 3, 37, 768), (3, 3, 70, 2048), (4, 300, 3, 1024),
                                      (5, 2, 17, 8192), (3, 2, 9, 3072), (1, 2, 7, 257), (2, 2, 5, 1001)])
@pytest.mark.parametrize("saved", [False, True])
def test_rmsnorm_against_oracle(cfg, B, T, D, saved):
    import torch
    from paper_2411_00999_amd import binding
    inp = workloads.make_inputs(cfg, B=B, T=T, D=D)
    inp.x += np.float32(0.5)                       # RMSNorm does not centre: give the rows a mean
    if inp.dtype == "bf16":
        inp.x = workloads.round_to_bf16(inp.x)
    eps = 1e-6
    ref = oracle.rms_bwd_pegn(inp.x, inp.dy, inp.gamma, eps, want_pe=False)
    x, dy, gamma = (pu.to_device(a, inp.dtype) for a in (inp.x, inp.dy, inp.gamma))
    y, rstd = binding.rms_fwd(x, gamma, eps)
    dx, dg, sg, big = binding.rms_bwd_ex(x, dy, gamma, eps, binding.PER_EXAMPLE, rstd=rstd if saved else None)
    torch.cuda.synchronize()
    bf = inp.dtype == "bf16"
    tol = pu.TOL_BF16 if bf else pu.TOL_F32
    y_ref, rstd_ref = oracle.rms_fwd(inp.x, inp.gamma, eps)
    pu.check_close("y", pu.to_host64(y), y_ref, tol, bf16_output=bf)
    np.testing.assert_allclose(pu.to_host64(rstd), rstd_ref, rtol=pu.TOL_F32)
    x64, dy64 = inp.x.reshape(-1, D).astype(np.float64), inp.dy.reshape(-1, D).astype(np.float64)
    term = float(np.sqrt(np.mean((rstd_ref.reshape(-1, 1) * dy64 * inp.gamma.astype(np.float64)) ** 2)))
    pu.check_close("dx", pu.to_host64(dx), ref["dx"], tol, bf16_output=bf, floor_rms=term)
    pu.check_close("dgamma", pu.to_host64(dg), ref["dgamma"], pu.TOL_SUMS)
    np.testing.assert_allclose(pu.to_host64(sg), ref["s_gamma"], rtol=pu.TOL_SUMS)
    np.testing.assert_allclose(pu.to_host64(big), ref["big_sq"], rtol=pu.TOL_SUMS)
    # plain call (no per-example outputs) gives the same dx and dgamma
    dx2, dg2, none_s, none_b = binding.rms_bwd_ex(x, dy, gamma, eps, 0)
    torch.cuda.synchronize()
    assert none_s is None and none_b is None
    pu.check_close("dgamma(plain)", pu.to_host64(dg2), ref["dgamma"], pu.TOL_SUMS)
    if not saved:
        assert torch.equal(dx, dx2)
    if B > 1:
        out = binding.gns_estimate(sg, big, float(B))
        torch.cuda.synchronize()
        _check_gns(out.cpu().numpy().astype(np.float64), oracle.gns_estimate(ref["s_gamma"], ref["big_sq"], float(B)), B)


# ------------------------------------------------------------------ estimator alone
@pytest.mark.parametrize("n_groups,B", [(1, 2), (2, 8), (96, 16), (3, 513)])
def test_gns_estimate_same_norms_both_sides(n_groups, B):
    import torch
    from paper_2411_00999_amd import binding
    rng = np.random.default_rng(n_groups * 1000 + B)
    mu = rng.standard_normal((n_groups, 1, 6)) * 0.7
    g = mu + rng.standard_normal((n_groups, B, 6))
    pe = np.sum((g / B) ** 2, -1).astype(np.float32)
    big = np.sum(g.mean(1) ** 2, -1).astype(np.float32)
    out = binding.gns_estimate(torch.from_numpy(pe).cuda(), torch.from_numpy(big).cuda(), float(B))
    torch.cuda.synchronize()
    want = oracle.gns_estimate(pe.astype(np.float64), big.astype(np.float64), float(B))
    keys = ("g_small_sq", "g_big_sq", "G2", "S", "B_simple")
    np.testing.assert_allclose(out.cpu().numpy(), [want[k] for k in keys], rtol=pu.TOL_GNS)


# ------------------------------------------------------------------ full sizes
def _sampled_dx_check(inp, res, n_rows=64, seed=0):
    """dx of a row depends on that row alone: check sampled rows one by one at any size."""
    rng = np.random.default_rng(seed)
    N = inp.B * inp.T
    rows = np.unique(np.concatenate([[0, N - 1], rng.integers(0, N, n_rows)]))
    x2, dy2 = inp.x.reshape(N, inp.D), inp.dy.reshape(N, inp.D)
    want = np.stack([oracle.ln_bwd_example(x2[r:r + 1], dy2[r:r + 1], inp.gamma, inp.eps)[0][0]
                     for r in rows])
    tol = pu.TOL_BF16 if inp.dtype == "bf16" else pu.TOL_F32
    pu.check_close("dx(sampled rows)", res["dx"].reshape(N, inp.D)[rows], want, tol,
                   bf16_output=inp.dtype == "bf16", floor_rms=pu.dx_term_rms(inp, rows))
    # property that holds for every row at any size: sum_d dx = 0 (up to output rounding)
    dx = res["dx"].reshape(N, inp.D)
    row_sum = np.abs(dx.sum(-1))
    budget = (2.0 ** -8 if inp.dtype == "bf16" else 2.0 ** -20) * np.abs(dx).sum(-1) / np.sqrt(inp.D) * 8 + 1e-30
    assert np.all(row_sum <= budget), float(np.max(row_sum / budget))


def test_more_than_2_to_31_elements():
    """Index arithmetic is 64-bit: B*T*D = 2^31 + 2*8192 elements per tensor (12 GiB for x, dy, dx).
    Inputs are drawn on the device (seeded) and copied to the host, so both sides read the same
    bf16 values; the oracle does the whole tensor for the sums and sampled rows for dx."""
    import torch
    from paper_2411_00999_amd import binding
    B, T, D = 4, 65537, 8192
    assert B * T * D > 2 ** 31
    gen = torch.Generator(device="cuda").manual_seed(2411)
    x = torch.empty((B, T, D), dtype=torch.bfloat16, device="cuda")
    dy = torch.empty((B, T, D), dtype=torch.bfloat16, device="cuda")
    for b in range(B):                                    # per example: bounds the fp32 temporaries
        x[b] = (torch.randn((T, D), generator=gen, device="cuda") * 1.5 + 0.25).to(torch.bfloat16)
        dy[b] = (torch.randn((T, D), generator=gen, device="cuda") * 1e-3).to(torch.bfloat16)
    gamma = (1.0 + 0.05 * torch.randn(D, generator=gen, device="cuda")).to(torch.bfloat16)
    eps = 1e-5
    dx, dg, db, sg, sb, big = binding.ln_bwd_pegn(x, dy, gamma, eps)
    torch.cuda.synchronize()
    g64 = gamma.float().cpu().numpy().astype(np.float64)
    dgamma, dbeta = np.zeros(D), np.zeros(D)
    s_gamma, s_beta = np.zeros(B), np.zeros(B)
    for b in range(B):                                    # the oracle, one example at a time
        xb = x[b].float().cpu().numpy().astype(np.float64)
        dyb = dy[b].float().cpu().numpy().astype(np.float64)
        _, gg, gb = oracle.ln_bwd_example(xb, dyb, g64, eps, want_dx=False)
        dgamma += gg
        dbeta += gb
        s_gamma[b], s_beta[b] = np.sum(gg * gg), np.sum(gb * gb)
        rows = np.unique(np.concatenate([[0, T - 1], np.random.default_rng(b).integers(0, T, 12)]))
        want = np.stack([oracle.ln_bwd_example(xb[r:r + 1], dyb[r:r + 1], g64, eps)[0][0] for r in rows])
        got = dx[b][torch.from_numpy(rows).cuda()].float().cpu().numpy().astype(np.float64)
        pu.check_close(f"dx[{b}] sampled rows", got, want, pu.TOL_BF16, bf16_output=True)
        del xb, dyb
    pu.check_close("dgamma", pu.to_host64(dg), dgamma, pu.TOL_SUMS)
    pu.check_close("dbeta", pu.to_host64(db), dbeta, pu.TOL_SUMS)
    np.testing.assert_allclose(pu.to_host64(sg), s_gamma, rtol=pu.TOL_SUMS)
    np.testing.assert_allclose(pu.to_host64(sb), s_beta, rtol=pu.TOL_SUMS)
    np.testing.assert_allclose(pu.to_host64(big), [np.sum(dgamma ** 2), np.sum(dbeta ** 2)], rtol=pu.TOL_SUMS)


@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_full_size_workloads(cfg):
    inp = workloads.make_inputs(cfg)
    ref = _oracle(inp, want_dx=False)
    res = pu.run_gpu(inp, saved_stats=(cfg == 3))
    pu.compare_with_oracle(inp, res, ref)
    _sampled_dx_check(inp, res, seed=cfg)
    got, want = _gns_both(res, ref, inp.B)
    _check_gns(got, want, inp.B)
    if cfg == 4:
        # half of the examples are copies of example 0: their norms coincide (up to the order
        # of the fp32 sums, which depends on where each example's sweep starts), and S equals
        # the closed form  [ n/2 |a-ubar|^2 + sum_i |u_i-ubar|^2 ] / (2n-1)
        n = inp.B // 2
        np.testing.assert_allclose(res["s_gamma"][:n], res["s_gamma"][0], rtol=2e-6)
        np.testing.assert_allclose(res["s_beta"][:n], res["s_beta"][0], rtol=2e-6)
        o = oracle.ln_bwd_pegn(inp.x, inp.dy, inp.gamma, inp.eps, want_dx=False)
        g = inp.B * np.concatenate([o["pe_gamma"], o["pe_beta"]], axis=1)
        a, u = g[0], g[n:]
        ubar = u.mean(0)
        closed = ((n / 2.0) * np.sum((a - ubar) ** 2) + np.sum((u - ubar) ** 2)) / (2 * n - 1)
        assert got[3] == pytest.approx(closed, rel=pu.TOL_GNS)


def test_full_size_headline_shape_in_fp32():
    """B=16 T=2048 D=2048 with fp32 storage, the launch configuration bench.py times (2048 chunks, several rounds
    of workgroups)."""
    from paper_2411_00999_amd import binding
    inp = workloads.make_inputs(3, dtype="f32")
    assert binding.plan_query(inp.B, inp.T, inp.D, binding.F32)["chunks"] == 2048
    ref = _oracle(inp, want_dx=False)
    res = pu.run_gpu(inp)
    pu.compare_with_oracle(inp, res, ref)
    _sampled_dx_check(inp, res, seed=33)
    got, want = _gns_both(res, ref, inp.B)
    _check_gns(got, want, inp.B)


# ------------------------------------------------------------------ GNS tracker: EMA, offline jackknife, schedule
def _records(g2, s):
    """[n,5] fp32 records with G2 and S in the places gns_estimate writes them."""
    rec = np.zeros((len(g2), 5), dtype=np.float32)
    rec[:, 2], rec[:, 3] = g2, s
    rec[:, 4] = rec[:, 3] / rec[:, 2]
    return rec


@pytest.mark.parametrize("n,alpha", [(1, 0.9), (3, 0.0), (300, 0.95), (1000, 0.999)])
def test_ema_tracker_against_oracle(n, alpha):
    import torch
    from oracle import gns_tracker_oracle as trk
    from paper_2411_00999_amd import binding
    rng = np.random.default_rng(workloads.BASE_SEED + n)
    state = torch.zeros((n, 3), dtype=torch.float64, device="cuda")
    ref = trk.ema_init(n)
    for step in range(25):
        rec = _records(rng.normal(2.0, 1.0, n), rng.normal(50.0, 20.0, n))
        smoothed = binding.gns_ema_update(state, torch.from_numpy(rec).cuda(), alpha)
        torch.cuda.synchronize()
        ref = trk.ema_update(ref, rec[:, 2].astype(np.float64), rec[:, 3].astype(np.float64), alpha)
        np.testing.assert_allclose(state.cpu().numpy(), ref, rtol=1e-13, atol=0)
        np.testing.assert_allclose(smoothed.cpu().numpy().astype(np.float64), trk.ema_read(ref), rtol=pu.TOL_F32)


def test_ema_tracker_follows_gns_estimate_records():
    """End to end on the device: per-example norms -> gns_estimate record -> smoothed estimate."""
    import torch
    from oracle import gns_tracker_oracle as trk
    from paper_2411_00999_amd import binding
    state = torch.zeros((1, 3), dtype=torch.float64, device="cuda")
    ref = trk.ema_init(1)
    for layer in range(4):
        inp = workloads.make_inputs(1, layer=layer, B=4, T=16, D=64, signal=True)
        gpu = pu.run_gpu(inp, pegn=True)
        dev = gpu["_dev"]
        rec = binding.gns_estimate(torch.stack([dev["sg"], dev["sb"]]), dev["big"], 4.0)
        smoothed = binding.gns_ema_update(state, rec.reshape(1, 5), 0.9)
        torch.cuda.synchronize()
        r = oracle.ln_bwd_pegn(inp.x, inp.dy, inp.gamma, workloads.EPS, want_dx=False, want_pe=False)
        est = oracle.gns_estimate(np.stack([r["s_gamma"], r["s_beta"]]), r["big_sq"], 4.0)
        ref = trk.ema_update(ref, [est["G2"]], [est["S"]], 0.9)
        np.testing.assert_allclose(smoothed.cpu().numpy().astype(np.float64), trk.ema_read(ref), rtol=1e-4)


@pytest.mark.parametrize("n", [2, 3, 17, 257, 2000])
def test_offline_jackknife_against_brute_force_oracle(n):
    import torch
    from oracle import gns_tracker_oracle as trk
    from paper_2411_00999_amd import binding
    rng = np.random.default_rng(workloads.BASE_SEED + 7 * n)
    rec = _records(rng.normal(3.0, 0.5, n), rng.normal(6.0, 2.0, n))
    out = binding.gns_offline(torch.from_numpy(rec).cuda())
    torch.cuda.synchronize()
    ref = trk.offline_gns(rec[:, 2].astype(np.float64), rec[:, 3].astype(np.float64))
    got = out.cpu().numpy().astype(np.float64)
    want = [ref[k] for k in ("mean_G2", "mean_S", "B_simple", "stderr", "B_simple_jack")]
    np.testing.assert_allclose(got, want, rtol=pu.TOL_F32)


def test_offline_jackknife_long_history_and_hand_example():
    import json
    import os
    import torch
    from oracle import gns_tracker_oracle as trk
    from paper_2411_00999_amd import binding
    rng = np.random.default_rng(workloads.BASE_SEED + 99)
    n = 300_001
    rec = _records(rng.normal(3.0, 0.5, n), rng.normal(6.0, 2.0, n))
    out = binding.gns_offline(torch.from_numpy(rec).cuda()).cpu().numpy().astype(np.float64)
    ref = trk.offline_gns_sums(rec[:, 2].astype(np.float64), rec[:, 3].astype(np.float64))
    np.testing.assert_allclose(out, [ref[k] for k in ("mean_G2", "mean_S", "B_simple", "stderr", "B_simple_jack")],
                               rtol=pu.TOL_F32)
    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "gns_tracker_hand_example.json")))["jackknife"]
    out = binding.gns_offline(torch.from_numpy(_records(g["G2"], g["S"])).cuda()).cpu().numpy()
    np.testing.assert_allclose(out, [2.0, 4.0, 2.0, np.sqrt(37.0) / 9.0, 19.0 / 9.0], rtol=1e-6)


def test_tracker_argument_errors():
    import torch
    from paper_2411_00999_amd import binding
    rec = torch.zeros((1, 5), dtype=torch.float32, device="cuda")
    with pytest.raises(binding.LnpegnError):
        binding.gns_offline(rec)                                   # n < 2
    st = torch.zeros((1, 3), dtype=torch.float64, device="cuda")
    for alpha in (1.0, -0.1, float("nan")):
        with pytest.raises(binding.LnpegnError):
            binding.gns_ema_update(st, rec, alpha)
    assert torch.count_nonzero(st).item() == 0


# ------------------------------------------------------------------ linear-layer per-example norms (Algorithm 1)
def _run_linear(x, g, dtype, w0=None):
    import torch
    from paper_2411_00999_amd import binding
    xd, gd = pu.to_device(x, dtype), pu.to_device(g, dtype)
    w = None if w0 is None else torch.from_numpy(w0.astype(np.float32)).cuda()
    w, s, big = binding.linear_pegn(xd, gd, w=w, accumulate=w0 is not None)
    torch.cuda.synchronize()
    return pu.to_host64(w), pu.to_host64(s), pu.to_host64(big)


def _check_linear(x, g, got, w0=None):
    from oracle import linear_pegn_oracle as lin
    ref = lin.linear_pegn(x, g)
    w_ref = ref["w"] if w0 is None else ref["w"] + w0.astype(np.float32).astype(np.float64)
    w, s, big = got
    pu.check_close("w", w, w_ref, pu.TOL_SUMS)
    np.testing.assert_allclose(s, ref["s"], rtol=pu.TOL_SUMS, err_msg="s")
    np.testing.assert_allclose(big, [np.sum(w_ref ** 2)], rtol=pu.TOL_SUMS, err_msg="big_sq")


@pytest.mark.parametrize("B,T,K,L", [
    (2, 64, 256, 128),        # exactly one tile, one stage
    (3, 70, 264, 136),        # ragged in T, K and L; examples split over workgroups
    (1, 1, 8, 8),             # smallest the matrix-core kernel takes
    (5, 200, 768, 768),       # hidden 768, several tiles
    (16, 33, 520, 1032),
    (2, 64, 4096, 2048),      # 256 tiles: no split over examples, totals written by the tile kernel
    (3, 129, 4104, 2056),     # the same with ragged edges
    (70, 16, 256, 128),       # more examples than the largest split
])
def test_linear_pegn_matrix_core_kernel(B, T, K, L):
    x, g = workloads.make_linear_inputs(B * 1000 + T, B, T, K, L, "bf16")
    _check_linear(x, g, _run_linear(x, g, "bf16"))


@pytest.mark.parametrize("B,T,K,L", [
    (2, 32, 256, 128),        # one tile, one fp32 stage (32 positions)
    (3, 70, 260, 132),        # ragged in T, K and L (multiples of 4, not of 8)
    (1, 1, 4, 4),
    (5, 96, 768, 768),
    (2, 64, 4096, 2048),      # no split over examples
    (3, 33, 4100, 2052),
])
def test_linear_pegn_matrix_core_kernel_fp32(B, T, K, L):
    x, g = workloads.make_linear_inputs(B * 1000 + T + 1, B, T, K, L, "f32")
    _check_linear(x, g, _run_linear(x, g, "f32"))
    if K * L < 1 << 20:
        w0 = np.random.default_rng(workloads.BASE_SEED + 80).normal(0, 1e-2, (K, L))
        _check_linear(x, g, _run_linear(x, g, "f32", w0=w0), w0=w0)


@pytest.mark.parametrize("B,T,K,L", [(3, 70, 264, 136), (2, 64, 4096, 2048)])
def test_linear_pegn_accumulates_into_the_weight_gradient(B, T, K, L):
    x, g = workloads.make_linear_inputs(77, B, T, K, L, "bf16")
    w0 = np.random.default_rng(workloads.BASE_SEED + 78).normal(0, 1e-2, (K, L))
    _check_linear(x, g, _run_linear(x, g, "bf16", w0=w0), w0=w0)


@pytest.mark.parametrize("dtype,B,T,K,L", [("f32", 3, 17, 50, 36), ("bf16", 2, 9, 100, 7), ("f32", 2, 64, 256, 128),
                                           ("f32", 1, 1, 1, 1)])
def test_linear_pegn_generic_kernel(dtype, B, T, K, L):
    x, g = workloads.make_linear_inputs(B * 1000 + K, B, T, K, L, dtype)
    _check_linear(x, g, _run_linear(x, g, dtype))
    w0 = np.random.default_rng(workloads.BASE_SEED + 79).normal(0, 1e-2, (K, L))
    _check_linear(x, g, _run_linear(x, g, dtype, w0=w0), w0=w0)


def test_linear_pegn_special_cases_and_estimate():
    import torch
    from paper_2411_00999_amd import binding
    B, T, K, L = 4, 96, 512, 256
    x, g = workloads.make_linear_inputs(5, B, T, K, L, "bf16", signal=1e-3)
    # identical examples: every s equal, w = B * w_0
    xi, gi = np.repeat(x[:1], B, 0), np.repeat(g[:1], B, 0)
    w, s, big = _run_linear(xi, gi, "bf16")
    np.testing.assert_allclose(s, s[0], rtol=1e-6)
    np.testing.assert_allclose(big[0], B * B * s[0], rtol=1e-5)
    # T = 1: the product form of Section 2.2
    x1, g1 = workloads.make_linear_inputs(6, 6, 1, 264, 136, "bf16")
    _, s1, _ = _run_linear(x1, g1, "bf16")
    np.testing.assert_allclose(s1, (x1[:, 0].astype(np.float64) ** 2).sum(1) * (g1[:, 0].astype(np.float64) ** 2).sum(1),
                               rtol=1e-5)
    # repeated calls are bitwise reproducible, and the norms feed the estimator (one group)
    xd, gd = pu.to_device(x, "bf16"), pu.to_device(g, "bf16")
    a = binding.linear_pegn(xd, gd)
    b = binding.linear_pegn(xd, gd)
    torch.cuda.synchronize()
    assert all(torch.equal(p, q) for p, q in zip(a, b))
    est = binding.gns_estimate(a[1], a[2], float(B)).cpu().numpy().astype(np.float64)
    from oracle import linear_pegn_oracle as lin
    ref = lin.linear_pegn(x, g)
    _check_gns(est, oracle.gns_estimate(ref["s"], [np.sum(ref["w"] ** 2)], float(B)), B)


@pytest.mark.parametrize("name", ["gpt111m_qkv", "gpt1p3b_up"])
def test_linear_pegn_full_size_sampled(name):
    """Full-size layers in the configuration the benchmark times.  The full [B,K,L] definition is out
    of the oracle's reach here, so: sampled entries of w' one by one, s[b] of two examples by the Gram
    form of Section 2.2 (pinned to the definition on the CPU), and big_sq against the w' it came with."""
    import torch
    from oracle import linear_pegn_oracle as lin
    from paper_2411_00999_amd import binding
    B, T, K, L = workloads.LINEAR_SHAPES[name]
    torch.manual_seed(workloads.BASE_SEED % (2 ** 31))
    # drawn on the device (the host generator would need minutes at this size), read back for the oracle
    xd = torch.randn((B, T, K), device="cuda").to(torch.bfloat16)
    gd = (torch.randn((B, T, L), device="cuda") * 1e-3 + torch.randn((1, T, L), device="cuda") * 1e-3).to(torch.bfloat16)
    w, s, big = binding.linear_pegn(xd, gd)
    torch.cuda.synchronize()
    rng = np.random.default_rng(workloads.BASE_SEED + 5)
    ks = np.concatenate([rng.integers(0, K, 60), [0, K - 1, 255, 256]])
    ls = np.concatenate([rng.integers(0, L, 60), [0, L - 1, 127, 128]])
    x_cols = xd[:, :, torch.from_numpy(ks).cuda()].float().cpu().numpy().astype(np.float64)     # [B,T,n]
    g_cols = gd[:, :, torch.from_numpy(ls).cuda()].float().cpu().numpy().astype(np.float64)
    want = lin.linear_pegn_entries(x_cols, g_cols, range(len(ks)), range(len(ks)))
    got = w[torch.from_numpy(ks).cuda(), torch.from_numpy(ls).cuda()].cpu().numpy().astype(np.float64)
    rms = float(torch.sqrt(torch.mean(w.double() ** 2)))
    assert np.all(np.abs(got - want) <= pu.TOL_SUMS * (np.abs(want) + rms)), np.max(np.abs(got - want)) / rms
    for b in (0, B - 1):
        ref = lin.gram_sq_norm(xd[b].float().cpu().numpy(), gd[b].float().cpu().numpy())
        assert float(s[b]) == pytest.approx(ref, rel=pu.TOL_SUMS), b
    assert float(big[0]) == pytest.approx(float(torch.sum(w.double() ** 2)), rel=pu.TOL_SUMS)


def test_linear_pegn_argument_errors():
    import torch
    from paper_2411_00999_amd import binding
    lib = binding.load()
    x = torch.zeros((2, 8, 16), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((16, 16), dtype=torch.float32, device="cuda")
    s = torch.zeros(2, dtype=torch.float32, device="cuda")
    ws = torch.zeros(lib.linear_pegn_workspace_bytes(2, 8, 16, 16, 1), dtype=torch.uint8, device="cuda")
    args = lambda **kw: [kw.get("x", x.data_ptr()), x.data_ptr(), w.data_ptr(), s.data_ptr(), None,
                         kw.get("B", 2), 8, 16, 16, kw.get("dt", 1), ws.data_ptr(), kw.get("wsb", ws.numel()),
                         kw.get("flags", 0), None]
    assert lib.linear_pegn(*args()) == 0
    assert lib.linear_pegn(*args(x=None)) == 1
    assert lib.linear_pegn(*args(B=0)) == 1
    assert lib.linear_pegn(*args(flags=1)) == 1
    assert lib.linear_pegn(*args(dt=7)) == 2
    assert lib.linear_pegn(*args(wsb=16)) == 3
    assert lib.linear_pegn_workspace_bytes(0, 8, 16, 16, 1) == 0
    torch.cuda.synchronize()


# ------------------------------------------------------------------ embedding-layer per-example norms (Appendix B)
def _run_embedding(ids, g, V, dtype, w0=None, int32=False):
    import torch
    from paper_2411_00999_amd import binding
    gd = pu.to_device(g, dtype)
    idd = torch.from_numpy(ids.astype(np.int32 if int32 else np.int64)).cuda()
    w = None if w0 is None else torch.from_numpy(w0.astype(np.float32)).cuda()
    w, s, big = binding.embedding_pegn(idd, gd, V, w=w, accumulate=w0 is not None)
    torch.cuda.synchronize()
    return pu.to_host64(w), pu.to_host64(s), pu.to_host64(big)


def _check_embedding(ids, g, V, got, w0=None):
    from oracle import embedding_pegn_oracle as emb
    ref = emb.embedding_pegn(ids, g, V)
    w_ref = ref["w"] if w0 is None else ref["w"] + w0.astype(np.float32).astype(np.float64)
    w, s, big = got
    pu.check_close("w", w, w_ref, pu.TOL_SUMS)
    absent = np.setdiff1d(np.arange(V), np.unique(ids))
    if w0 is None and absent.size:
        assert not w[absent].any(), "rows of absent ids must be exactly zero"
    np.testing.assert_allclose(s, ref["s"], rtol=pu.TOL_SUMS, err_msg="s")
    np.testing.assert_allclose(big, [np.sum(w_ref ** 2)], rtol=pu.TOL_SUMS, err_msg="big_sq")


@pytest.mark.parametrize("dtype,B,T,D,V", [
    ("bf16", 4, 128, 768, 1000),      # several column blocks, a ragged last one
    ("bf16", 3, 70, 2048, 50257),     # GPT-2 vocabulary, most rows absent
    ("f32", 2, 33, 264, 97),
    ("bf16", 2, 9, 100, 7),           # D % 8 != 0: element loads
    ("f32", 1, 1, 1, 1),
    ("bf16", 16, 64, 512, 31),        # few ids: long runs per id, many examples per id
])
def test_embedding_pegn_against_oracle(dtype, B, T, D, V):
    ids, g = workloads.make_embedding_inputs(B * 100 + T, B, T, D, V, dtype)
    _check_embedding(ids, g, V, _run_embedding(ids, g, V, dtype))
    _check_embedding(ids, g, V, _run_embedding(ids, g, V, dtype, int32=True))
    w0 = np.random.default_rng(workloads.BASE_SEED + 81).normal(0, 1e-2, (V, D))
    _check_embedding(ids, g, V, _run_embedding(ids, g, V, dtype, w0=w0), w0=w0)


@pytest.mark.parametrize("dtype,B,T,D,V", [("bf16", 4, 128, 768, 1000), ("bf16", 3, 70, 2048, 50257), ("f32", 2, 33, 264, 97),
                                           ("bf16", 2, 9, 100, 7), ("bf16", 16, 64, 512, 31)])
def test_embedding_pegn_presorted_matches_the_sorting_call(dtype, B, T, D, V):
    """ids sorted beforehand (embedding_sort_ids, as a forward pass would): the same kernels on the same order, so
    the results are bitwise those of embedding_pegn, overwrite and accumulate; out-of-range ids included."""
    import torch
    from oracle import embedding_pegn_oracle as emb
    from paper_2411_00999_amd import binding
    ids, g = workloads.make_embedding_inputs(B * 100 + T + 7, B, T, D, V, dtype)
    gd = pu.to_device(g, dtype)
    idd = torch.from_numpy(ids).cuda()
    sk, sp = binding.embedding_sort_ids(idd, V)
    torch.cuda.synchronize()
    # the order itself: stable sort by id of the positions 0..n-1
    order = np.argsort(ids.reshape(-1), kind="stable")
    np.testing.assert_array_equal(sp.cpu().numpy(), order.astype(np.int32))
    np.testing.assert_array_equal(sk.cpu().numpy(), ids.reshape(-1)[order].astype(np.int32))
    for rep in range(2):                        # twice on one workspace: nothing is left behind
        want = binding.embedding_pegn(idd, gd, V)
        got = binding.embedding_pegn_presorted(sk, sp, gd, V)
        torch.cuda.synchronize()
        for a, b, name in zip(got, want, ("w", "s", "big_sq")):
            assert torch.equal(a, b), name
    _check_embedding(ids, g, V, tuple(pu.to_host64(t) for t in got))
    w0 = torch.from_numpy(np.random.default_rng(3).normal(0, 1e-2, (V, D)).astype(np.float32)).cuda()
    want = binding.embedding_pegn(idd, gd, V, w=w0.clone(), accumulate=True)
    got = binding.embedding_pegn_presorted(sk, sp, gd, V, w=w0.clone(), accumulate=True)
    torch.cuda.synchronize()
    for a, b in zip(got, want):
        assert torch.equal(a, b)
    # ids outside [0, V) are skipped by both calls
    bad = ids.copy()
    bad[0, 0], bad[-1, -1] = V, -3
    bd = torch.from_numpy(bad).cuda()
    sk2, sp2 = binding.embedding_sort_ids(bd, V)
    want = binding.embedding_pegn(bd, gd, V)
    got = binding.embedding_pegn_presorted(sk2, sp2, gd, V)
    torch.cuda.synchronize()
    for a, b in zip(got, want):
        assert torch.equal(a, b)
    keep = np.ones(ids.shape, bool)
    keep[0, 0] = keep[-1, -1] = False
    ref = emb.embedding_pegn(np.where(keep, ids, 0), g * keep[..., None], V)
    pu.check_close("w", pu.to_host64(got[0]), ref["w"], pu.TOL_SUMS)
    np.testing.assert_allclose(pu.to_host64(got[1]), ref["s"], rtol=pu.TOL_SUMS)


@pytest.mark.parametrize("B,T", [(1, 2048), (3, 2049), (16, 2048), (5, 5000), (64, 2048), (70, 2048)])
def test_embedding_sort_sizes_around_the_tile_boundaries(B, T):
    """One tile, a ragged second tile, the benchmark's 16 tiles, the largest batch our own sort takes (64 tiles)
    and one beyond it (the library's sort): the order is the stable sort by id, and the whole call matches."""
    import torch
    from paper_2411_00999_amd import binding
    V, D = 1000, 8
    ids, g = workloads.make_embedding_inputs(B + T, B, T, D, V, "f32")
    ids[0, : min(T, 7)] = [V, -1, 0, V - 1, 2 ** 31 - 1, -2 ** 31, 5][: min(T, 7)]      # out of range and the edges
    for int32 in (False, True):
        idd = torch.from_numpy(ids.astype(np.int32 if int32 else np.int64)).cuda()
        sk, sp = binding.embedding_sort_ids(idd, V)
        torch.cuda.synchronize()
        key = np.where((ids >= 0) & (ids < V), ids, V).reshape(-1)
        order = np.argsort(key, kind="stable")
        np.testing.assert_array_equal(sp.cpu().numpy(), order.astype(np.int32))
        np.testing.assert_array_equal(sk.cpu().numpy(), key[order].astype(np.int32))
    gd = pu.to_device(g, "f32")
    w, s, big = binding.embedding_pegn(idd, gd, V)
    w2, s2, big2 = binding.embedding_pegn_presorted(sk, sp, gd, V)
    torch.cuda.synchronize()
    assert torch.equal(w, w2) and torch.equal(s, s2) and torch.equal(big, big2)
    from oracle import embedding_pegn_oracle as emb
    keep = (ids >= 0) & (ids < V)
    ref = emb.embedding_pegn(np.where(keep, ids, 0), g * keep[..., None], V)
    pu.check_close("w", pu.to_host64(w), ref["w"], pu.TOL_SUMS)
    np.testing.assert_allclose(pu.to_host64(s), ref["s"], rtol=pu.TOL_SUMS)


def test_embedding_pegn_special_cases():
    import torch
    from paper_2411_00999_amd import binding
    B, T, D, V = 4, 96, 512, 300
    ids, g = workloads.make_embedding_inputs(9, B, T, D, V, "bf16")
    g64 = g.astype(np.float64)
    # one id throughout: s_b = |sum_t g_bt|^2; all ids distinct in an example: s_b = sum_t |g_bt|^2
    _, s_same, _ = _run_embedding(np.full((B, T), 5), g, V, "bf16")
    np.testing.assert_allclose(s_same, (g64.sum(1) ** 2).sum(1), rtol=1e-5)
    distinct = np.stack([np.random.default_rng(b).permutation(V)[:T] for b in range(B)])
    _, s_dist, _ = _run_embedding(distinct, g, V, "bf16")
    np.testing.assert_allclose(s_dist, (g64 ** 2).sum((1, 2)), rtol=1e-5)
    # ids outside [0,V) are skipped: the same result as without those positions' gradients
    bad = ids.copy()
    bad[:, ::7] = -3
    bad[:, 3::11] = V + 5
    g_masked = g.copy()
    g_masked[(bad < 0) | (bad >= V)] = 0.0
    w_bad, s_bad, big_bad = _run_embedding(bad, g, V, "bf16")
    ok = np.where((bad < 0) | (bad >= V), 0, bad)
    _check_embedding(ok, g_masked, V, (w_bad, s_bad, big_bad))
    # bitwise reproducible, and the norms feed the estimator
    gd, idd = pu.to_device(g, "bf16"), torch.from_numpy(ids).cuda()
    a = binding.embedding_pegn(idd, gd, V)
    b = binding.embedding_pegn(idd, gd, V)
    torch.cuda.synchronize()
    assert all(torch.equal(p, q) for p, q in zip(a, b))
    est = binding.gns_estimate(a[1], a[2], float(B)).cpu().numpy().astype(np.float64)
    from oracle import embedding_pegn_oracle as emb
    ref = emb.embedding_pegn(ids, g, V)
    _check_gns(est, oracle.gns_estimate(ref["s"], [np.sum(ref["w"] ** 2)], float(B)), B)


@pytest.mark.parametrize("dtype,D", [("bf16", 512), ("f32", 264), ("bf16", 100)])
def test_embedding_pegn_long_runs(dtype, D):
    """Runs longer than one piece: an id that fills one example and occurs nowhere else (one run, several
    pieces), an id that fills most of every example, and ordinary ids between them."""
    B, T, V = 5, 150, 400
    rng = np.random.default_rng(workloads.BASE_SEED + 83)
    _, g = workloads.make_embedding_inputs(83, B, T, D, V, dtype)
    ids = rng.integers(10, V, (B, T))
    ids[1, :] = 3                                   # one run of 150 rows, the id's only one
    ids[:, 20:131] = np.where(ids[:, 20:131] == 3, 4, 7)   # 111-row runs of id 7 in every example ...
    ids[1, 20:131] = 3                              # ... but example 1 stays id 3 throughout
    ids[2, 5:70:2] = 9                              # an id scattered inside one example: one run of 33 rows
    _check_embedding(ids, g, V, _run_embedding(ids, g, V, dtype))
    w0 = rng.normal(0, 1e-2, (V, D))
    _check_embedding(ids, g, V, _run_embedding(ids, g, V, dtype, w0=w0), w0=w0)


def test_embedding_pegn_two_threads_two_streams():
    """Calls from two host threads on two streams of one device share the library's side stream: every call must
    still give the single-call result bit for bit."""
    import threading
    import torch
    from paper_2411_00999_amd import binding
    B, T, D, V = 4, 256, 512, 3000
    cases = []
    for seed in (91, 92):
        ids, g = workloads.make_embedding_inputs(seed, B, T, D, V, "bf16")
        idd, gd = torch.from_numpy(ids).cuda(), pu.to_device(g, "bf16")
        ref = binding.embedding_pegn(idd, gd, V)
        torch.cuda.synchronize()
        cases.append((idd, gd, ref))
    results, errors = [None, None], []

    def work(k):
        try:
            st = torch.cuda.Stream()
            idd, gd, _ = cases[k]
            outs = []
            with torch.cuda.stream(st):
                for _ in range(20):
                    outs.append(binding.embedding_pegn(idd, gd, V, stream=st))
            st.synchronize()
            results[k] = outs
        except Exception as e:                      # surfaced in the main thread below
            errors.append(e)

    threads = [threading.Thread(target=work, args=(k,)) for k in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for k in range(2):
        for out in results[k]:
            assert all(torch.equal(a, b) for a, b in zip(out, cases[k][2]))


def test_embedding_pegn_argument_errors():
    import torch
    from paper_2411_00999_amd import binding
    lib = binding.load()
    ids = torch.zeros((2, 8), dtype=torch.int32, device="cuda")
    g = torch.zeros((2, 8, 16), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((5, 16), dtype=torch.float32, device="cuda")
    s = torch.zeros(2, dtype=torch.float32, device="cuda")
    nb = lib.embedding_pegn_workspace_bytes(2, 8, 16, 5)
    assert nb > 0
    ws = torch.zeros(nb, dtype=torch.uint8, device="cuda")
    args = lambda **kw: [kw.get("ids", ids.data_ptr()), 0, g.data_ptr(), w.data_ptr(), s.data_ptr(), None,
                         kw.get("B", 2), 8, 16, 5, kw.get("dt", 1), ws.data_ptr(), kw.get("wsb", ws.numel()),
                         kw.get("flags", 0), None]
    assert lib.embedding_pegn(*args()) == 0
    assert lib.embedding_pegn(*args(ids=None)) == 1
    assert lib.embedding_pegn(*args(B=0)) == 1
    assert lib.embedding_pegn(*args(flags=2)) == 1
    assert lib.embedding_pegn(*args(dt=9)) == 2
    assert lib.embedding_pegn(*args(wsb=64)) == 3
    assert lib.embedding_pegn_workspace_bytes(2, 8, 16, 0) == 0
    torch.cuda.synchronize()


# ------------------------------------------------------------------ the streaming yardstick is a real copy / xor
def test_stream_probe_modes():
    import torch
    from paper_2411_00999_amd import binding
    lib = binding.load()
    n = 4096 * 5 + 4 * 37                      # int32 words: whole workgroups and a ragged tail of 16-byte vectors
    g = torch.Generator(device="cpu").manual_seed(7)
    a = torch.randint(-2**31, 2**31 - 1, (n,), dtype=torch.int32, generator=g).cuda()
    b = torch.randint(-2**31, 2**31 - 1, (n,), dtype=torch.int32, generator=g).cuda()
    for mode, want in ((0, a), (1, a ^ b), (2, a ^ b)):
        out = torch.full_like(a, 12345)
        binding.stream_probe(a, b, out, mode)
        torch.cuda.synchronize()
        assert torch.equal(out, want), f"mode {mode}"
    out = torch.zeros_like(a)
    assert lib.lnpegn_stream_probe(a.data_ptr(), b.data_ptr(), out.data_ptr(), n * 4, 3, None) == 1
    assert lib.lnpegn_stream_probe(a.data_ptr(), None, out.data_ptr(), n * 4, 2, None) == 1
    assert lib.lnpegn_stream_probe(a.data_ptr(), b.data_ptr(), out.data_ptr(), n * 4 - 8, 2, None) == 1
    torch.cuda.synchronize()
