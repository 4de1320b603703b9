"""The pieces together on a small network: per-example gradient norms of every LayerNorm, linear and
embedding parameter from the library's kernels, combined by gns_estimate, against the same quantities
obtained the slow way -- one separate autograd backward per example on the CPU in fp64 (Section 2.1:
B_small = 1, B_big = B; Section 3: the 1/B^2 correction for a mean-reduced loss)."""
import numpy as np
import pytest

import oracle
import parity_util as pu
from paper_2411_00999_amd import workloads

pytestmark = pytest.mark.gpu


def _model_and_data(B, T, D, H, V, seed):
    import torch
    g = torch.Generator().manual_seed(seed)
    P = dict(
        emb=torch.randn(V, D, generator=g, dtype=torch.float64) * 0.5,
        g1=1.0 + 0.1 * torch.randn(D, generator=g, dtype=torch.float64),
        b1=0.1 * torch.randn(D, generator=g, dtype=torch.float64),
        w1=torch.randn(D, H, generator=g, dtype=torch.float64) / D ** 0.5,
        w2=torch.randn(H, D, generator=g, dtype=torch.float64) / H ** 0.5,
        g2=1.0 + 0.1 * torch.randn(D, generator=g, dtype=torch.float64),
        b2=0.1 * torch.randn(D, generator=g, dtype=torch.float64),
        w3=torch.randn(D, V, generator=g, dtype=torch.float64) / D ** 0.5,
    )
    ids = torch.randint(0, V, (B, T), generator=g)
    targets = torch.randint(0, V, (B, T), generator=g)
    return P, ids, targets


def _forward(P, ids, targets, keep):
    """Returns the per-example losses [B]; keep(name, tensor) is called on every activation the
    kernels need (inputs of the layers, retaining their gradients)."""
    import torch
    import torch.nn.functional as F
    eps = workloads.EPS
    h0 = keep("h0", P["emb"][ids])
    x1 = keep("ln1_out", F.layer_norm(h0, h0.shape[-1:], P["g1"], P["b1"], eps))
    a1 = keep("l1_out", x1 @ P["w1"])
    z = keep("l2_in", F.gelu(a1))
    a2 = keep("l2_out", z @ P["w2"])
    h1 = keep("ln2_in", h0 + a2)
    x2 = keep("ln2_out", F.layer_norm(h1, h1.shape[-1:], P["g2"], P["b2"], eps))
    logits = keep("l3_out", x2 @ P["w3"])
    B, T, V = logits.shape
    return F.cross_entropy(logits.reshape(B * T, V), targets.reshape(B * T), reduction="none").reshape(B, T).mean(1)


@pytest.mark.parametrize("B,T,D,H,V", [(4, 12, 32, 64, 50), (6, 5, 16, 24, 11)])
def test_network_noise_scale_matches_per_example_autograd(B, T, D, H, V):
    import torch
    from paper_2411_00999_amd import binding
    P, ids, targets = _model_and_data(B, T, D, H, V, seed=B * 100 + T)
    names = list(P)

    # ---- the slow way: one backward per example
    per_ex = []
    for b in range(B):
        Pb = {k: v.clone().requires_grad_(True) for k, v in P.items()}
        loss_b = _forward(Pb, ids[b:b + 1], targets[b:b + 1], lambda n, t: t)[0]
        grads = torch.autograd.grad(loss_b, [Pb[k] for k in names])
        per_ex.append(torch.cat([gr.reshape(-1) for gr in grads]))
    per_ex = torch.stack(per_ex)                                   # gradients of L_b, [B, n_params]
    g_small_sq = float((per_ex ** 2).sum(1).mean())               # B_small = 1
    g_big_sq = float((per_ex.mean(0) ** 2).sum())                 # gradient of the batch loss mean_b L_b
    want_G2, want_S, want_B = oracle.gns_from_norms(g_big_sq, g_small_sq, float(B), 1.0)

    # ---- one batch backward, activations and output gradients captured
    acts = {}

    def keep(name, t):
        t.retain_grad()
        acts[name] = t
        return t
    Pg = {k: v.clone().requires_grad_(True) for k, v in P.items()}
    _forward(Pg, ids, targets, keep).mean().backward()             # mean-reduced loss: dy carries 1/B
    dev = lambda t: t.detach().to(torch.float32).contiguous().cuda()
    eps = workloads.EPS
    s_groups, big_groups, checks = [], [], []

    def ln(x_name, out_name, gamma, pg, pb):
        dx, dg, db, sg, sb, big = binding.ln_bwd_pegn(dev(acts[x_name]), dev(acts[out_name].grad), dev(gamma), eps)
        s_groups.extend([sg, sb])
        big_groups.extend([big[0:1], big[1:2]])
        checks.extend([(dg, Pg[pg].grad), (db, Pg[pb].grad), (dx, None)])
    ln("h0", "ln1_out", P["g1"], "g1", "b1")
    ln("ln2_in", "ln2_out", P["g2"], "g2", "b2")
    for x_name, out_name, pw in (("ln1_out", "l1_out", "w1"), ("l2_in", "l2_out", "w2"), ("ln2_out", "l3_out", "w3")):
        w, s, big = binding.linear_pegn(dev(acts[x_name]), dev(acts[out_name].grad))
        s_groups.append(s)
        big_groups.append(big)
        checks.append((w, Pg[pw].grad))
    w, s, big = binding.embedding_pegn(ids.cuda(), dev(acts["h0"].grad), V)
    s_groups.append(s)
    big_groups.append(big)
    checks.append((w, Pg["emb"].grad))
    est = binding.gns_estimate(torch.stack(s_groups), torch.cat(big_groups), float(B))
    torch.cuda.synchronize()

    for got, ref in checks:                                        # the batch gradients themselves
        if ref is not None:
            pu.check_close("batch gradient", pu.to_host64(got), ref.numpy(), 1e-4)
    got = est.cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(got[0], g_small_sq, rtol=1e-4)
    np.testing.assert_allclose(got[1], g_big_sq, rtol=1e-4)
    np.testing.assert_allclose(got[3], want_S, rtol=1e-4)
    kappa = pu.gns_condition(B, g_big_sq, g_small_sq)
    np.testing.assert_allclose(got[2], want_G2, rtol=max(1e-4, 8 * kappa * 2.0 ** -23))
    np.testing.assert_allclose(got[4], want_B, rtol=2 * max(1e-4, 8 * kappa * 2.0 ** -23))
