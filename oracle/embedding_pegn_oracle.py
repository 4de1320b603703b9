"""TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT PATH.

Slow fp64 definition of what the embedding-layer per-example gradient-norm computation of Appendix B
(embedding-layer algorithm) must produce.  An embedding layer copies row ids[b,t] of its table to
output position (b,t); the gradient of example b's loss with respect to the table is therefore the
scatter-add of that example's output gradients by id,

    w_b[v,:] = sum over the positions t of example b with ids[b,t] == v of g[b,t,:]      [V,D]

and the quantities wanted are  s[b] = ||w_b||_F^2  (raw: the mean over b and the B^2 factor belong to
the estimator, gns_estimate with pe_scale = B)  and  w' = sum_b w_b.  The code below is that sentence:
a loop over (b,t) adding one row at a time into example b's own [V,D] array, which is formed on
purpose.  No one-hot tensor, no matrix product, no library step.  Nothing here is imported by the HIP
package.
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
        w_b = np.zeros((V, D))                       # example b's own table gradient
        for t in range(T):
            w_b[int(ids[b, t])] += g[b, t]           # the row that position (b,t) read
        s[b] = np.sum(w_b * w_b)
        w += w_b
        if want_pe:
            pe[b] = w_b
    return dict(w=w, s=s, pe=pe)
