"""Pins of the CPU oracle against things other than itself.

Each test checks the oracle against what the paper and the mathematics fix:
a hand-worked exact example, finite differences of the forward, a library
autograd of each example alone, closed forms, invariants and a Monte-Carlo
check of the estimators' unbiasedness.  None of these run on a GPU.
"""
import json
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_case(seed, B, T, D, dy_std=1.0, offset=0.0):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((B, T, D)) * rng.uniform(0.5, 2.0, (B, T, 1)) + offset
    dy = rng.standard_normal((B, T, D)) * dy_std
    gamma = 1.0 + 0.3 * rng.standard_normal(D)
    beta = 0.1 * rng.standard_normal(D)
    return x, dy, gamma, beta


# ---------------------------------------------------------------- hand-worked example
def test_hand_worked_example_exact():
    """Exact rationals derived by hand (tests/golden/ln_pegn_hand_example.json)."""
    with open(os.path.join(GOLDEN, "ln_pegn_hand_example.json")) as f:
        g = json.load(f)
    x, dy = np.array(g["x"], float), np.array(g["dy"], float)
    gamma = np.array(g["gamma"], float)
    e = g["expected"]
    mean, rstd = oracle.ln_stats(x, g["eps"])
    np.testing.assert_allclose(mean, e["mean"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(rstd, e["rstd"], rtol=1e-15)
    o = oracle.ln_bwd_pegn(x, dy, gamma, g["eps"])
    for key in ("dx", "pe_gamma", "pe_beta", "s_gamma", "s_beta", "dgamma", "dbeta", "big_sq"):
        np.testing.assert_allclose(o[key], np.array(e[key], float), rtol=1e-14, atol=1e-14, err_msg=key)
    est = oracle.gns_estimate(np.stack([o["s_gamma"], o["s_beta"]]), o["big_sq"], e["gns_pe_scale"])
    for key in ("g_small_sq", "g_big_sq", "G2", "S", "B_simple"):
        assert est[key] == pytest.approx(e[key], rel=1e-13), key


def test_hand_worked_forward():
    with open(os.path.join(GOLDEN, "ln_pegn_hand_example.json")) as f:
        g = json.load(f)
    y = oracle.ln_fwd(np.array(g["x"], float), np.array(g["gamma"], float), np.array(g["beta_fwd"], float),
                      g["eps"])
    np.testing.assert_allclose(y, np.array(g["expected"]["y_with_beta_fwd"], float), rtol=1e-14, atol=1e-14)


def test_forward_matches_library():
    import torch
    import torch.nn.functional as F
    x, _, gamma, beta = _rand_case(41, 3, 5, 37, offset=-2.0)
    y = oracle.ln_fwd(x, gamma, beta, 1e-5)
    want = F.layer_norm(torch.tensor(x), (37,), torch.tensor(gamma), torch.tensor(beta), 1e-5).numpy()
    np.testing.assert_allclose(y, want, rtol=1e-12, atol=1e-13)


def test_gradient_accumulation_is_the_big_batch():
    """A micro-batches of B examples, loss averaged over all A*B examples: summing the micro-batch
    gradients and concatenating the per-example norms is the same as one batch of A*B examples,
    with B_big = A*B and pe_scale = A*B in the estimator."""
    A, B, T, D = 3, 4, 5, 24
    x, dy, gamma, _ = _rand_case(43, A * B, T, D)
    whole = oracle.ln_bwd_pegn(x, dy, gamma, 1e-5)
    dgamma, dbeta = np.zeros(D), np.zeros(D)
    sg, sb = [], []
    for a in range(A):
        part = oracle.ln_bwd_pegn(x[a * B:(a + 1) * B], dy[a * B:(a + 1) * B], gamma, 1e-5)
        dgamma += part["dgamma"]
        dbeta += part["dbeta"]
        sg.append(part["s_gamma"])
        sb.append(part["s_beta"])
    np.testing.assert_allclose(dgamma, whole["dgamma"], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dbeta, whole["dbeta"], rtol=1e-12, atol=1e-14)
    np.testing.assert_array_equal(np.concatenate(sg), whole["s_gamma"])
    big = np.array([np.sum(dgamma ** 2), np.sum(dbeta ** 2)])
    est_acc = oracle.gns_estimate(np.stack([np.concatenate(sg), np.concatenate(sb)]), big, pe_scale=A * B)
    est_whole = oracle.gns_estimate(np.stack([whole["s_gamma"], whole["s_beta"]]), whole["big_sq"],
                                    pe_scale=A * B)
    for k in est_whole:
        assert est_acc[k] == pytest.approx(est_whole[k], rel=1e-10)


# ---------------------------------------------------------------- P1 finite differences
def _loss(x, dy, gamma, beta, eps):
    return float(np.sum(dy * oracle.ln_fwd(x, gamma, beta, eps)))


def test_finite_differences_dx_dgamma_dbeta_and_per_example():
    B, T, D, eps, h = 2, 3, 5, 1e-5, 1e-6
    x, dy, gamma, beta = _rand_case(11, B, T, D)
    o = oracle.ln_bwd_pegn(x, dy, gamma, eps)

    fd_dx = np.zeros_like(x)
    for idx in np.ndindex(*x.shape):
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        fd_dx[idx] = (_loss(xp, dy, gamma, beta, eps) - _loss(xm, dy, gamma, beta, eps)) / (2 * h)
    np.testing.assert_allclose(o["dx"], fd_dx, rtol=1e-6, atol=1e-8)

    fd_g, fd_b = np.zeros(D), np.zeros(D)
    fd_pg, fd_pb = np.zeros((B, D)), np.zeros((B, D))
    for k in range(D):
        for arr, fd, fdp in ((gamma, fd_g, fd_pg), (beta, fd_b, fd_pb)):
            ap, am = arr.copy(), arr.copy()
            ap[k] += h
            am[k] -= h
            args_p = (ap, beta) if arr is gamma else (gamma, ap)
            args_m = (am, beta) if arr is gamma else (gamma, am)
            fd[k] = (_loss(x, dy, *args_p, eps) - _loss(x, dy, *args_m, eps)) / (2 * h)
            for b in range(B):   # the loss of example b alone
                fdp[b, k] = (_loss(x[b], dy[b], *args_p, eps) - _loss(x[b], dy[b], *args_m, eps)) / (2 * h)
    np.testing.assert_allclose(o["dgamma"], fd_g, rtol=1e-7, atol=1e-8)
    np.testing.assert_allclose(o["dbeta"], fd_b, rtol=1e-7, atol=1e-8)
    np.testing.assert_allclose(o["pe_gamma"], fd_pg, rtol=1e-7, atol=1e-8)
    np.testing.assert_allclose(o["pe_beta"], fd_pb, rtol=1e-7, atol=1e-8)


# ---------------------------------------------------------------- P2 / P11 library autograd
def _torch_ln_grads(x, dy, gamma, beta, eps):
    import torch
    import torch.nn.functional as F
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    gt = torch.tensor(gamma, dtype=torch.float64, requires_grad=True)
    bt = torch.tensor(beta, dtype=torch.float64, requires_grad=True)
    y = F.layer_norm(xt, (x.shape[-1],), gt, bt, eps)
    (y * torch.tensor(dy)).sum().backward()
    return xt.grad.numpy(), gt.grad.numpy(), bt.grad.numpy()


@pytest.mark.parametrize("shape", [(3, 7, 33), (5, 1, 16), (1, 9, 64), (4, 6, 1)])
def test_library_autograd_each_example_alone_and_whole_batch(shape):
    B, T, D = shape
    eps = 1e-5
    x, dy, gamma, beta = _rand_case(7 + D, B, T, D, offset=3.0)
    o = oracle.ln_bwd_pegn(x, dy, gamma, eps)
    # whole batch at once: dgamma/dbeta/dx (sum over b of separate backwards == one batch backward)
    dx, dg, db = _torch_ln_grads(x, dy, gamma, beta, eps)
    np.testing.assert_allclose(o["dx"], dx, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(o["dgamma"], dg, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(o["dbeta"], db, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(o["big_sq"], [np.sum(dg ** 2), np.sum(db ** 2)], rtol=1e-10, atol=1e-20)
    # each example alone
    for b in range(B):
        dxb, dgb, dbb = _torch_ln_grads(x[b], dy[b], gamma, beta, eps)
        np.testing.assert_allclose(o["pe_gamma"][b], dgb, rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(o["pe_beta"][b], dbb, rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(o["dx"][b], dxb, rtol=1e-9, atol=1e-11)
        assert o["s_gamma"][b] == pytest.approx(np.sum(dgb ** 2), rel=1e-10, abs=1e-20)
        assert o["s_beta"][b] == pytest.approx(np.sum(dbb ** 2), rel=1e-10)
        _, gg, gb = oracle.ln_bwd_example(x[b], dy[b], gamma, eps, want_dx=False)
        np.testing.assert_array_equal(gg, o["pe_gamma"][b])
        np.testing.assert_array_equal(gb, o["pe_beta"][b])


def test_stats_match_library():
    x, _, _, _ = _rand_case(3, 2, 5, 48, offset=-7.0)
    mean, rstd = oracle.ln_stats(x, 1e-5)
    np.testing.assert_allclose(mean, x.mean(-1), rtol=1e-13)
    np.testing.assert_allclose(rstd, 1.0 / np.sqrt(x.var(-1) + 1e-5), rtol=1e-13)


# ---------------------------------------------------------------- P3 B = 1
def test_batch_of_one_norm_equals_big_norm():
    x, dy, gamma, beta = _rand_case(5, 1, 12, 40)
    o = oracle.ln_bwd_pegn(x, dy, gamma, 1e-5)
    _, dg, db = _torch_ln_grads(x, dy, gamma, beta, 1e-5)
    assert o["s_gamma"][0] == pytest.approx(np.sum(dg ** 2), rel=1e-11)
    assert o["s_beta"][0] == pytest.approx(np.sum(db ** 2), rel=1e-11)
    assert o["s_gamma"][0] == pytest.approx(o["big_sq"][0], rel=1e-14)
    assert o["s_beta"][0] == pytest.approx(o["big_sq"][1], rel=1e-14)


# ---------------------------------------------------------------- P4 row invariants of dx
@pytest.mark.parametrize("eps", [0.0, 1e-5, 1e-2])
def test_dx_row_invariants(eps):
    B, T, D = 3, 4, 96
    x, dy, gamma, _ = _rand_case(21, B, T, D, offset=1.5)
    o = oracle.ln_bwd_pegn(x, dy, gamma, eps)
    mu = x.mean(-1, keepdims=True)
    rstd = 1.0 / np.sqrt(x.var(-1, keepdims=True) + eps)
    xhat = (x - mu) * rstd
    scale = np.abs(o["dx"]).sum(-1)
    # sum_d dx = 0 exactly (up to rounding) because sum_d xhat = 0
    assert np.all(np.abs(o["dx"].sum(-1)) <= 1e-13 * scale)
    # sum_d dx*xhat = D * c1 * eps * rstd^3, which vanishes only for eps = 0
    c1 = (dy * gamma * xhat).mean(-1)
    want = D * c1 * eps * rstd[..., 0] ** 3
    got = (o["dx"] * xhat).sum(-1)
    np.testing.assert_allclose(got, want, rtol=1e-9, atol=1e-13 * scale.max())


def test_d2_eps0_dx_vanishes():
    """D = 2, eps = 0: xhat is (+-1, -+1) whatever x is, so the output cannot move and dx = 0."""
    rng = np.random.default_rng(2)
    x = rng.standard_normal((2, 5, 2))
    dy = rng.standard_normal((2, 5, 2))
    o = oracle.ln_bwd_pegn(x, dy, np.array([1.3, -0.7]), 0.0)
    assert np.max(np.abs(o["dx"])) < 1e-12 * np.max(np.abs(dy)) / np.min(np.abs(x[..., 0] - x[..., 1]))


def test_constant_row_is_finite():
    """sigma^2 = 0: rstd = 1/sqrt(eps), xhat = 0, everything finite."""
    B, T, D, eps = 2, 3, 8, 1e-5
    x, dy, gamma, _ = _rand_case(9, B, T, D)
    x[0, 1] = 4.25
    o = oracle.ln_bwd_pegn(x, dy, gamma, eps)
    assert all(np.all(np.isfinite(v)) for v in o.values())
    dyh = dy[0, 1] * gamma
    np.testing.assert_allclose(o["dx"][0, 1], (dyh - dyh.mean()) / np.sqrt(eps), rtol=1e-12)


# ---------------------------------------------------------------- P5 identical examples
def test_identical_examples_have_zero_noise():
    B, T, D = 6, 5, 24
    x, dy, gamma, _ = _rand_case(13, 1, T, D)
    x, dy = np.repeat(x, B, 0), np.repeat(dy, B, 0)
    o = oracle.ln_bwd_pegn(x, dy, gamma, 1e-5)
    est = oracle.gns_estimate(np.stack([o["s_gamma"], o["s_beta"]]), o["big_sq"], pe_scale=B)
    big = o["big_sq"].sum()
    assert abs(est["S"]) <= 1e-12 * big
    assert est["G2"] == pytest.approx(big, rel=1e-12)
    assert abs(est["B_simple"]) <= 1e-12


# ---------------------------------------------------------------- P6 sample-covariance identity
def test_estimators_equal_sample_covariance_trace():
    """With B_small = 1 and g_b = B * g'_b:  S = trace of the unbiased sample covariance of the
    g_b, and G2 = |mean g|^2 - S/B."""
    B, T, D = 7, 4, 20
    x, dy, gamma, _ = _rand_case(17, B, T, D)
    o = oracle.ln_bwd_pegn(x, dy, gamma, 1e-5)
    g = B * np.concatenate([o["pe_gamma"], o["pe_beta"]], axis=1)      # [B, 2D]
    gbar = g.mean(0)
    S = np.sum((g - gbar) ** 2) / (B - 1)
    G2 = np.sum(gbar ** 2) - S / B
    est = oracle.gns_estimate(np.stack([o["s_gamma"], o["s_beta"]]), o["big_sq"], pe_scale=B)
    assert est["S"] == pytest.approx(S, rel=1e-10)
    assert est["G2"] == pytest.approx(G2, rel=1e-8, abs=1e-12 * np.sum(gbar ** 2))
    assert est["g_big_sq"] == pytest.approx(np.sum(gbar ** 2), rel=1e-12)
    # one group at a time is the same function
    one = oracle.gns_estimate(o["s_gamma"], o["big_sq"][:1], pe_scale=B)
    gg = B * o["pe_gamma"]
    assert one["S"] == pytest.approx(np.sum((gg - gg.mean(0)) ** 2) / (B - 1), rel=1e-10)


# ---------------------------------------------------------------- P7 half the examples identical
def test_half_identical_examples_closed_form():
    from paper_2411_00999_amd import workloads
    inp = workloads.make_inputs(4, B=16, T=8, D=64)
    B = inp.B
    n = B // 2
    o = oracle.ln_bwd_pegn(inp.x, inp.dy, inp.gamma, inp.eps)
    g = B * np.concatenate([o["pe_gamma"], o["pe_beta"]], axis=1)
    np.testing.assert_array_equal(g[:n], np.repeat(g[:1], n, 0))      # the copies really are copies
    a, u = g[0], g[n:]
    ubar = u.mean(0)
    S_closed = ((n / 2.0) * np.sum((a - ubar) ** 2) + np.sum((u - ubar) ** 2)) / (2 * n - 1)
    est = oracle.gns_estimate(np.stack([o["s_gamma"], o["s_beta"]]), o["big_sq"], pe_scale=B)
    assert est["S"] == pytest.approx(S_closed, rel=1e-10)


# ---------------------------------------------------------------- P8 T = 1 (2-D) special case
def test_T1_reduces_to_elementwise_product_form():
    """With one position per example the per-example squared norm of an elementwise affine is
    sum_k xhat^2 dy^2 (the 2-D trick of Section 2.2 applied to a diagonal weight)."""
    B, D, eps = 9, 50, 1e-5
    x, dy, gamma, _ = _rand_case(19, B, 1, D)
    o = oracle.ln_bwd_pegn(x, dy, gamma, eps)
    xhat = (x - x.mean(-1, keepdims=True)) / np.sqrt(x.var(-1, keepdims=True) + eps)
    np.testing.assert_allclose(o["s_gamma"], np.sum(xhat[:, 0] ** 2 * dy[:, 0] ** 2, -1), rtol=1e-12)
    np.testing.assert_allclose(o["s_beta"], np.sum(dy[:, 0] ** 2, -1), rtol=1e-12)


# ---------------------------------------------------------------- P9 equivariances
def test_equivariances():
    B, T, D, eps = 4, 6, 32, 1e-5
    x, dy, gamma, _ = _rand_case(23, B, T, D)
    o = oracle.ln_bwd_pegn(x, dy, gamma, eps)
    a, c = 3.5, -11.0
    o_dy = oracle.ln_bwd_pegn(x, a * dy, gamma, eps)
    np.testing.assert_allclose(o_dy["dx"], a * o["dx"], rtol=1e-12)
    np.testing.assert_allclose(o_dy["s_gamma"], a * a * o["s_gamma"], rtol=1e-12)
    np.testing.assert_allclose(o_dy["s_beta"], a * a * o["s_beta"], rtol=1e-12)
    e0 = oracle.gns_estimate(np.stack([o["s_gamma"], o["s_beta"]]), o["big_sq"], B)
    e1 = oracle.gns_estimate(np.stack([o_dy["s_gamma"], o_dy["s_beta"]]), o_dy["big_sq"], B)
    assert e1["B_simple"] == pytest.approx(e0["B_simple"], rel=1e-9)
    # affine change of x with eps scaled alike leaves xhat alone
    o_x = oracle.ln_bwd_pegn(a * x + c, dy, gamma, a * a * eps)
    np.testing.assert_allclose(o_x["dgamma"], o["dgamma"], rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(o_x["s_gamma"], o["s_gamma"], rtol=1e-9)
    np.testing.assert_allclose(o_x["dx"], o["dx"] / a, rtol=1e-8, atol=1e-12)
    # permuting examples permutes s; permuting positions inside an example leaves s and dgamma alone
    perm = np.array([2, 0, 3, 1])
    o_p = oracle.ln_bwd_pegn(x[perm], dy[perm], gamma, eps)
    np.testing.assert_allclose(o_p["s_gamma"], o["s_gamma"][perm], rtol=1e-13)
    np.testing.assert_allclose(o_p["dx"], o["dx"][perm], rtol=1e-13)
    tperm = np.random.default_rng(1).permutation(T)
    o_t = oracle.ln_bwd_pegn(x[:, tperm], dy[:, tperm], gamma, eps)
    np.testing.assert_allclose(o_t["s_gamma"], o["s_gamma"], rtol=1e-12)
    np.testing.assert_allclose(o_t["dgamma"], o["dgamma"], rtol=1e-11, atol=1e-13)
    # beta never enters the backward; gamma scales dx only through dy*gamma
    assert np.all(o["dbeta"] == dy.sum((0, 1))) or np.allclose(o["dbeta"], dy.sum((0, 1)), rtol=1e-13)


# ---------------------------------------------------------------- estimator algebra + P10 Monte Carlo
def test_eq4_eq5_exact_on_noise_model_moments():
    """If |G_B|^2 takes its expectation |G|^2 + tr(Sigma)/B at both batch sizes, Eq. 4 and Eq. 5
    return |G|^2 and tr(Sigma) exactly, for any pair of batch sizes."""
    G2, trS = 3.7, 11.3
    for b_big, b_small in ((8, 1), (64, 4), (7, 3), (1000, 10)):
        big = G2 + trS / b_big
        small = G2 + trS / b_small
        g2, s, bs = oracle.gns_from_norms(big, small, b_big, b_small)
        assert g2 == pytest.approx(G2, rel=1e-12)
        assert s == pytest.approx(trS, rel=1e-12)
        assert bs == pytest.approx(trS / G2, rel=1e-12)
    with pytest.raises(ValueError):
        oracle.gns_from_norms(1.0, 2.0, 4, 4)
    with pytest.raises(ValueError):
        oracle.gns_estimate(np.ones((1, 1)), np.ones(1), 1.0)


def test_monte_carlo_unbiasedness_true_gns_one():
    """The simulation setting of Section 2.1 (Figure 2): gradients ~ N(G, Sigma) with
    tr(Sigma)/|G|^2 = 1.  Means of S and G2 over many draws approach tr(Sigma) and |G|^2."""
    rng = np.random.default_rng(1234)
    d, B, trials = 12, 8, 20000
    G = rng.standard_normal(d)
    G *= 2.0 / np.linalg.norm(G)                       # |G|^2 = 4
    sig = rng.uniform(0.5, 1.5, d)
    sig *= np.sqrt(4.0 / np.sum(sig ** 2))            # tr(Sigma) = 4
    S_vals, G2_vals = np.empty(trials), np.empty(trials)
    for i in range(trials):
        g = G + sig * rng.standard_normal((B, d))      # per-example gradients of the sum loss
        raw = np.sum((g / B) ** 2, -1)                 # what a mean-reduced loss hands back
        big = np.sum(g.mean(0) ** 2)
        est = oracle.gns_estimate(raw, [big], pe_scale=B)
        S_vals[i], G2_vals[i] = est["S"], est["G2"]
    for vals, want in ((S_vals, 4.0), (G2_vals, 4.0)):
        stderr = vals.std(ddof=1) / np.sqrt(trials)
        assert abs(vals.mean() - want) < 3.5 * stderr, (vals.mean(), want, stderr)
    # ratio of the means (what smoothing before the ratio approaches) is the true noise scale
    assert S_vals.mean() / G2_vals.mean() == pytest.approx(1.0, abs=0.05)


def test_monte_carlo_general_batch_sizes():
    rng = np.random.default_rng(99)
    d, b_big, b_small, trials = 6, 12, 3, 20000
    G = np.full(d, 1.0)
    trS = 5.0
    sig = np.sqrt(trS / d)
    S_vals, G2_vals = np.empty(trials), np.empty(trials)
    for i in range(trials):
        g = G + sig * rng.standard_normal((b_big, d))
        big = np.sum(g.mean(0) ** 2)
        small = np.mean(np.sum(g.reshape(b_big // b_small, b_small, d).mean(1) ** 2, -1))
        G2_vals[i], S_vals[i], _ = oracle.gns_from_norms(big, small, b_big, b_small)
    for vals, want in ((S_vals, trS), (G2_vals, float(d))):
        stderr = vals.std(ddof=1) / np.sqrt(trials)
        assert abs(vals.mean() - want) < 3.5 * stderr


# ---------------------------------------------------------------- P12 magnitude sanity on workloads
def test_workload_magnitudes():
    from paper_2411_00999_amd import workloads
    inp = workloads.make_inputs(2, B=4, T=64, D=768)
    o = oracle.ln_bwd_pegn(inp.x, inp.dy, inp.gamma, inp.eps, want_dx=False)
    expect = inp.D * inp.T * (1e-3) ** 2          # E s_beta[b] for iid dy of std 1e-3
    assert np.all(np.abs(o["s_beta"] / expect - 1.0) < 0.2)
    assert np.all(np.abs(o["s_gamma"] / expect - 1.0) < 0.2)


def test_threads_do_not_change_results():
    x, dy, gamma, _ = _rand_case(31, 6, 5, 40)
    a = oracle.ln_bwd_pegn(x, dy, gamma, 1e-5, nthreads=1)
    b = oracle.ln_bwd_pegn(x, dy, gamma, 1e-5, nthreads=4)
    for k in a:
        np.testing.assert_array_equal(a[k], b[k])


# ---------------------------------------------------------------- RMSNorm variant
def test_rms_hand_worked_example_exact():
    with open(os.path.join(GOLDEN, "rms_pegn_hand_example.json")) as f:
        g = json.load(f)
    x, dy, gamma = np.array(g["x"], float), np.array(g["dy"], float), np.array(g["gamma"], float)
    e = g["expected"]
    y, rstd = oracle.rms_fwd(x, gamma, g["eps"])
    np.testing.assert_allclose(rstd, e["rstd"], rtol=1e-15)
    np.testing.assert_allclose(y, np.array(e["y"], float), rtol=1e-14, atol=1e-14)
    o = oracle.rms_bwd_pegn(x, dy, gamma, g["eps"])
    for key in ("dx", "pe_gamma", "s_gamma", "dgamma", "big_sq"):
        np.testing.assert_allclose(o[key], np.array(e[key], float), rtol=1e-14, atol=1e-14, err_msg=key)
    est = oracle.gns_estimate(o["s_gamma"], o["big_sq"], e["gns_pe_scale"])
    for key in ("g_small_sq", "g_big_sq", "G2", "S", "B_simple"):
        assert est[key] == pytest.approx(e[key], rel=1e-13), key


def _torch_rms_grads(x, dy, gamma, eps):
    import torch
    import torch.nn.functional as F
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    gt = torch.tensor(gamma, dtype=torch.float64, requires_grad=True)
    y = F.rms_norm(xt, (x.shape[-1],), gt, eps)
    (y * torch.tensor(dy)).sum().backward()
    return y.detach().numpy(), xt.grad.numpy(), gt.grad.numpy()


@pytest.mark.parametrize("shape", [(3, 6, 40), (4, 1, 8), (1, 5, 1)])
def test_rms_library_autograd_each_example_and_whole_batch(shape):
    B, T, D = shape
    eps = 1e-6
    x, dy, gamma, _ = _rand_case(61 + D, B, T, D, offset=0.7)
    o = oracle.rms_bwd_pegn(x, dy, gamma, eps)
    y, dx, dg = _torch_rms_grads(x, dy, gamma, eps)
    np.testing.assert_allclose(oracle.rms_fwd(x, gamma, eps)[0], y, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(o["dx"], dx, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(o["dgamma"], dg, rtol=1e-10, atol=1e-12)
    assert o["big_sq"][0] == pytest.approx(np.sum(dg ** 2), rel=1e-10)
    for b in range(B):
        _, dxb, dgb = _torch_rms_grads(x[b], dy[b], gamma, eps)
        np.testing.assert_allclose(o["pe_gamma"][b], dgb, rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(o["dx"][b], dxb, rtol=1e-9, atol=1e-11)
        assert o["s_gamma"][b] == pytest.approx(np.sum(dgb ** 2), rel=1e-10)


def test_rms_finite_differences_and_invariants():
    B, T, D, eps, h = 2, 3, 6, 1e-6, 1e-6
    x, dy, gamma, _ = _rand_case(67, B, T, D, offset=0.3)
    o = oracle.rms_bwd_pegn(x, dy, gamma, eps)
    loss = lambda xx, gg: float(np.sum(dy * oracle.rms_fwd(xx, gg, eps)[0]))
    fd = np.zeros_like(x)
    for idx in np.ndindex(*x.shape):
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        fd[idx] = (loss(xp, gamma) - loss(xm, gamma)) / (2 * h)
    np.testing.assert_allclose(o["dx"], fd, rtol=1e-6, atol=1e-8)
    # sum_d dx*xhat = D*c1*eps*rstd^3: the row gradient is orthogonal to xhat when eps = 0
    o0 = oracle.rms_bwd_pegn(x, dy, gamma, 0.0)
    xhat = x / np.sqrt(np.mean(x * x, -1, keepdims=True))
    assert np.max(np.abs((o0["dx"] * xhat).sum(-1))) < 1e-12 * np.abs(o0["dx"]).sum(-1).max()
    # a centred input makes RMSNorm and LayerNorm agree (mean = 0), gamma gradients included
    xc = x - x.mean(-1, keepdims=True)
    ln = oracle.ln_bwd_pegn(xc, dy, gamma, eps)
    rm = oracle.rms_bwd_pegn(xc, dy, gamma, eps)
    np.testing.assert_allclose(rm["dgamma"], ln["dgamma"], rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(rm["s_gamma"], ln["s_gamma"], rtol=1e-10)
