"""TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT PATH.

Slow fp64 definition of the embedding-layer simultaneous per-example gradient-norm computation
(Appendix B, embedding-layer algorithm): for token ids x [B,T] in [0,V) and gradients g [B,T,D] of the
loss with respect to the embedding outputs,

    step 1   o = onehot(x, V)                               [B,T,V]
    step 2   w_b[v,d] = sum_t o[b,t,v] * g[b,t,d]           (per-example weight gradient [V,D])
    step 3   s_w[b]   = sum_{v,d} w_b[v,d]^2
    step 4   w'[v,d]  = sum_b w_b[v,d]

Step 5 (mean over b, times B^2) is the estimator's business (gns_estimate with pe_scale = B): s_w is
returned raw.  The one-hot tensor and the per-example [V,D] gradient are formed on purpose -- that is
the definition; one matrix product per example is the only library step.  Nothing here is imported by
the HIP package.
"""
from __future__ import annotations

import numpy as np


def embedding_pegn(ids, g, V: int, want_pe: bool = False) -> dict:
    """ids [B,T] integers in [0,V), g [B,T,D] -> dict(w [V,D], s [B], pe [B,V,D] or None), float64."""
    ids = np.asarray(ids)
    g = np.asarray(g, dtype=np.float64)
    if ids.ndim != 2 or g.ndim != 3 or ids.shape != g.shape[:2]:
        raise ValueError("ids must be [B,T] and g [B,T,D]")
    if not np.issubdtype(ids.dtype, np.integer) or ids.min(initial=0) < 0 or ids.max(initial=0) >= V:
        raise ValueError("ids must be integers in [0,V)")
    B, T, D = g.shape
    w = np.zeros((V, D))
    s = np.zeros(B)
    pe = np.zeros((B, V, D)) if want_pe else None
    for b in range(B):
        onehot = np.zeros((T, V))
        onehot[np.arange(T), ids[b]] = 1.0          # step 1 for this example
        w_b = onehot.T @ g[b]                        # step 2
        s[b] = np.sum(w_b * w_b)                     # step 3
        w += w_b                                     # step 4
        if want_pe:
            pe[b] = w_b
    return dict(w=w, s=s, pe=pe)
