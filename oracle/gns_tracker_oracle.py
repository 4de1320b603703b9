"""TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT PATH.

Slow fp64 definitions of what is done with the per-step estimates of Eq. 4 (G2, the squared norm of
the true gradient) and Eq. 5 (S, the trace of the per-example covariance) after they are computed:

* online:  both estimators are smoothed separately with an exponential moving average and only then
  divided (Section 4.2, "GNS Correlates Between Layer Types": every GNS figure smooths both
  estimators before taking the ratio);
* offline: the per-step estimates are averaged with a plain mean and the uncertainty of the ratio
  of means is measured with the jackknife for ratio estimators (Figure 2 caption; Appendix A, last
  paragraph);
* the linear batch-size schedule of Section 5.1, realised through the number of accumulation steps.

Plain numpy / Python loops, fp64 (Python integers for the schedule), no blocking and no reordering.
Nothing here is imported by the HIP package.
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------------------- online: EMA
def ema_init(n: int) -> np.ndarray:
    """Fresh state for n tracked groups: rows (m_G2, m_S, w), all zero."""
    return np.zeros((n, 3), dtype=np.float64)


def ema_update(state: np.ndarray, g2, s, alpha: float) -> np.ndarray:
    """One step of  m <- alpha*m + (1-alpha)*v  for v = G2 and v = S, and the same recurrence on the
    constant 1 (w), which is the total weight the zero-initialised average has seen: w = 1-alpha^t."""
    g2 = np.atleast_1d(np.asarray(g2, dtype=np.float64))
    s = np.atleast_1d(np.asarray(s, dtype=np.float64))
    new = np.empty_like(state)
    for i in range(state.shape[0]):
        new[i, 0] = alpha * state[i, 0] + (1.0 - alpha) * g2[i]
        new[i, 1] = alpha * state[i, 1] + (1.0 - alpha) * s[i]
        new[i, 2] = alpha * state[i, 2] + (1.0 - alpha) * 1.0
    return new


def ema_read(state: np.ndarray) -> np.ndarray:
    """Rows (G2_smooth, S_smooth, B_simple_smooth): the averages divided by their weight, and Eq. 3
    applied to the smoothed pair (the weight cancels in the ratio)."""
    out = np.empty_like(state)
    with np.errstate(divide="ignore", invalid="ignore"):
        for i in range(state.shape[0]):
            out[i, 0] = state[i, 0] / state[i, 2]
            out[i, 1] = state[i, 1] / state[i, 2]
            out[i, 2] = np.float64(state[i, 1]) / np.float64(state[i, 0])
    return out


def ema_series(g2, s, alpha: float) -> np.ndarray:
    """Smoothed (G2, S, B_simple) after each of the t steps of one group -> [t,3]."""
    g2 = np.asarray(g2, dtype=np.float64)
    s = np.asarray(s, dtype=np.float64)
    st = ema_init(1)
    out = np.empty((g2.shape[0], 3))
    for t in range(g2.shape[0]):
        st = ema_update(st, g2[t:t + 1], s[t:t + 1], alpha)
        out[t] = ema_read(st)[0]
    return out


# ----------------------------------------------------------------------------- offline: mean + jackknife
def offline_gns(g2, s) -> dict:
    """Ratio of means and its delete-one jackknife, by actually deleting each step and recomputing.

    R = mean(S)/mean(G2);  R_(i) = the same with step i left out;  Rbar = mean_i R_(i);
    stderr = sqrt((n-1)/n * sum_i (R_(i)-Rbar)^2);  bias-corrected  R_jack = n*R - (n-1)*Rbar.
    """
    g2 = np.asarray(g2, dtype=np.float64)
    s = np.asarray(s, dtype=np.float64)
    n = g2.shape[0]
    if n < 2 or s.shape[0] != n:
        raise ValueError("the jackknife needs n >= 2 paired estimates")
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = np.mean(s) / np.mean(g2)
        loo = np.empty(n)
        for i in range(n):
            loo[i] = np.mean(np.delete(s, i)) / np.mean(np.delete(g2, i))
        rbar = np.mean(loo)
        stderr = np.sqrt((n - 1.0) / n * np.sum((loo - rbar) ** 2))
    return dict(mean_G2=float(np.mean(g2)), mean_S=float(np.mean(s)), B_simple=float(ratio),
                stderr=float(stderr), B_simple_jack=float(n * ratio - (n - 1.0) * rbar))


def offline_gns_sums(g2, s) -> dict:
    """The same quantities with the left-out means written as (sum - element)/(n-1): identical
    mathematics, O(n), for histories too long to delete from one by one."""
    g2 = np.asarray(g2, dtype=np.float64)
    s = np.asarray(s, dtype=np.float64)
    n = g2.shape[0]
    if n < 2 or s.shape[0] != n:
        raise ValueError("the jackknife needs n >= 2 paired estimates")
    with np.errstate(divide="ignore", invalid="ignore"):
        sum_g, sum_s = np.sum(g2), np.sum(s)
        ratio = sum_s / sum_g
        loo = (sum_s - s) / (sum_g - g2)
        rbar = np.mean(loo)
        stderr = np.sqrt((n - 1.0) / n * np.sum((loo - rbar) ** 2))
    return dict(mean_G2=float(sum_g / n), mean_S=float(sum_s / n), B_simple=float(ratio),
                stderr=float(stderr), B_simple_jack=float(n * ratio - (n - 1.0) * rbar))


# ----------------------------------------------------------------------------- batch-size schedule
def linear_accum_steps(tokens_seen: int, ramp_tokens: int, accum_final: int) -> int:
    """Section 5.1: the batch size grows linearly with the tokens processed until it reaches the
    original batch size, and is varied through the number of accumulation steps.  With A_final
    steps at the original size:  A = ceil(A_final * tokens/ramp), kept within [1, A_final]."""
    if tokens_seen < 0 or ramp_tokens < 0 or accum_final < 1:
        raise ValueError("bad schedule arguments")
    if ramp_tokens == 0 or tokens_seen >= ramp_tokens:
        return accum_final
    a = -((-accum_final * tokens_seen) // ramp_tokens)
    return max(1, min(accum_final, a))
