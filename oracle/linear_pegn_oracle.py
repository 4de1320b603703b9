"""TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT PATH.

Slow fp64 definition of what the linear-layer per-example gradient-norm computation of Section 3
(Algorithm 1) must produce.  A linear layer maps x[b,t,:] (K features) to x[b,t,:] @ W (L features);
with g [B,T,L] the gradient of the loss with respect to its outputs, the gradient of example b's loss
with respect to W is the sum over that example's positions of the outer products of input and output
gradient,

    w_b = sum_t outer(x[b,t,:], g[b,t,:]) = x_b^T g_b                                     [K,L]

(every middle dimension is flattened into t), and the quantities wanted are  s[b] = ||w_b||_F^2  (raw:
the mean over b and the B^2 factor belong to the estimator, gns_estimate with pe_scale = B, as for the
LayerNorm path)  and  w' = sum_b w_b.  The per-example matrix is formed on purpose -- that is the
definition; one matrix product per example is the only library step, and linear_pegn_entries and
gram_sq_norm below reach the same numbers without it.  Nothing here is imported by the HIP package.
"""
from __future__ import annotations

import numpy as np


def linear_pegn(x, g, want_pe: bool = False) -> dict:
    """x [B,T,K], g [B,T,L] -> dict(w [K,L], s [B], pe [B,K,L] or None), all float64."""
    x = np.asarray(x, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    if x.ndim != 3 or g.ndim != 3 or x.shape[:2] != g.shape[:2]:
        raise ValueError("x must be [B,T,K] and g [B,T,L] with the same B and T")
    B, T, K = x.shape
    L = g.shape[2]
    w = np.zeros((K, L))
    s = np.zeros(B)
    pe = np.zeros((B, K, L)) if want_pe else None
    for b in range(B):
        w_b = x[b].T @ g[b]                 # example b's own weight gradient
        s[b] = np.sum(w_b * w_b)
        w += w_b
        if want_pe:
            pe[b] = w_b
    return dict(w=w, s=s, pe=pe)


def linear_pegn_entries(x, g, ks, ls) -> np.ndarray:
    """Selected entries of the batch gradient, one by one: w'[k,l] = sum_b sum_t x[b,t,k] * g[b,t,l] for each pair
    (ks[i], ls[i]).  For shapes whose full [K,L] result is out of the oracle's reach."""
    x = np.asarray(x)
    g = np.asarray(g)
    out = np.empty(len(ks))
    for i, (k, l) in enumerate(zip(ks, ls)):
        out[i] = np.sum(x[:, :, k].astype(np.float64) * g[:, :, l].astype(np.float64))
    return out


def gram_sq_norm(x_b, g_b) -> float:
    """||w_b||_F^2 for ONE example without forming w_b: the three-dimensional form of Section 2.2,
    n_b^2 = <X_b X_b^T, G_b G_b^T>_F  (X_b [T,K], G_b [T,L]; O(T^2) memory)."""
    x_b = np.asarray(x_b, dtype=np.float64)
    g_b = np.asarray(g_b, dtype=np.float64)
    return float(np.sum((x_b @ x_b.T) * (g_b @ g_b.T)))
