"""Pins for oracle/gns_tracker_oracle.py: hand-worked rationals, closed forms, textbook identities,
brute force and Monte Carlo -- none of them re-types the oracle's own formula.  The last test plants
mistakes in a copy of the oracle's source and checks that each one fails a pin."""
import json
import os
import types
from fractions import Fraction

import numpy as np
import pytest

from oracle import gns_tracker_oracle as trk

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "gns_tracker_hand_example.json")))


def _fr(v):
    return float(Fraction(v))


# ----------------------------------------------------------------------------- EMA
def test_ema_hand_example(o=trk):
    g = GOLD["ema"]
    st = o.ema_init(1)
    for t in range(2):
        st = o.ema_update(st, [g["G2"][t]], [g["S"][t]], g["alpha"])
        np.testing.assert_allclose(st[0], [g["m_G2"][t], g["m_S"][t], g["w"][t]], rtol=1e-15)
        np.testing.assert_allclose(o.ema_read(st)[0], [_fr(g["G2_smooth"][t]), _fr(g["S_smooth"][t]),
                                                       _fr(g["B_simple_smooth"][t])], rtol=1e-15)


def test_ema_constant_sequence_is_reproduced_at_every_step(o=trk):
    out = o.ema_series(np.full(40, 3.25), np.full(40, -7.5), 0.9)
    np.testing.assert_allclose(out[:, 0], 3.25, rtol=1e-14)
    np.testing.assert_allclose(out[:, 1], -7.5, rtol=1e-14)
    np.testing.assert_allclose(out[:, 2], -7.5 / 3.25, rtol=1e-14)


@pytest.mark.parametrize("alpha", [0.0, 0.3, 0.9, 0.999])
def test_ema_equals_geometric_weighted_mean(alpha, o=trk):
    rng = np.random.default_rng(5)
    g2, s = rng.normal(2.0, 1.0, 60), rng.normal(5.0, 2.0, 60)
    out = o.ema_series(g2, s, alpha)
    for t in (1, 2, 7, 60):
        wts = np.array([alpha ** (t - 1 - k) if alpha > 0 or k == t - 1 else 0.0 for k in range(t)])
        wg, ws = np.dot(wts, g2[:t]) / wts.sum(), np.dot(wts, s[:t]) / wts.sum()
        np.testing.assert_allclose(out[t - 1], [wg, ws, ws / wg], rtol=1e-12)


def test_ema_limits(o=trk):
    rng = np.random.default_rng(6)
    g2, s = rng.normal(2.0, 1.0, 9), rng.normal(5.0, 2.0, 9)
    np.testing.assert_allclose(o.ema_series(g2, s, 0.0)[:, :2], np.stack([g2, s], 1), rtol=1e-15)   # no memory
    np.testing.assert_allclose(o.ema_series(g2, s, 0.7)[0, :2], [g2[0], s[0]], rtol=1e-14)            # first step
    # alpha -> 1 approaches the plain running mean
    out = o.ema_series(g2, s, 1.0 - 1e-9)
    np.testing.assert_allclose(out[-1, :2], [g2.mean(), s.mean()], rtol=1e-6)


def test_ema_groups_are_independent(o=trk):
    st = o.ema_init(3)
    st = o.ema_update(st, [1.0, 2.0, 3.0], [4.0, 5.0, 6.0], 0.8)
    st = o.ema_update(st, [2.0, 2.0, 2.0], [1.0, 1.0, 1.0], 0.8)
    for i, (a, b) in enumerate([(1.0, 4.0), (2.0, 5.0), (3.0, 6.0)]):
        one = o.ema_update(o.ema_update(o.ema_init(1), [a], [b], 0.8), [2.0], [1.0], 0.8)
        np.testing.assert_array_equal(st[i], one[0])


# ----------------------------------------------------------------------------- jackknife
def test_jackknife_hand_example(o=trk):
    g = GOLD["jackknife"]
    for fn in (o.offline_gns, o.offline_gns_sums):
        r = fn(g["G2"], g["S"])
        assert r["B_simple"] == pytest.approx(_fr(g["B_simple"]), rel=1e-15)
        assert r["stderr"] ** 2 == pytest.approx(_fr(g["stderr_squared"]), rel=1e-13)
        assert r["B_simple_jack"] == pytest.approx(_fr(g["B_simple_jack"]), rel=1e-13)
        assert r["mean_G2"] == pytest.approx(2.0) and r["mean_S"] == pytest.approx(4.0)


def test_jackknife_of_a_plain_mean_is_the_textbook_standard_error(o=trk):
    """With a constant denominator the ratio is a sample mean, for which the delete-one jackknife
    gives exactly s/sqrt(n) and no bias correction."""
    rng = np.random.default_rng(7)
    s = rng.normal(3.0, 2.0, 25)
    for fn in (o.offline_gns, o.offline_gns_sums):
        r = fn(np.full(25, 4.0), s)
        assert r["B_simple"] == pytest.approx(s.mean() / 4.0, rel=1e-14)
        assert r["stderr"] == pytest.approx(s.std(ddof=1) / np.sqrt(25) / 4.0, rel=1e-10)
        assert r["B_simple_jack"] == pytest.approx(r["B_simple"], rel=1e-10)


def test_jackknife_two_forms_agree_and_symmetries(o=trk):
    rng = np.random.default_rng(8)
    g2, s = rng.normal(2.0, 0.5, 200), rng.normal(6.0, 3.0, 200)
    a, b = o.offline_gns(g2, s), o.offline_gns_sums(g2, s)
    for k in a:
        assert a[k] == pytest.approx(b[k], rel=1e-9), k
    perm = rng.permutation(200)
    p = o.offline_gns(g2[perm], s[perm])
    scaled = o.offline_gns(4.0 * g2, 0.5 * s)
    for k in ("B_simple", "stderr", "B_simple_jack"):
        assert p[k] == pytest.approx(a[k], rel=1e-10)
        assert scaled[k] == pytest.approx(a[k] / 8.0, rel=1e-10)
    # pairing matters: shifting S against G2 changes the answer when they are correlated
    with pytest.raises(ValueError):
        o.offline_gns([1.0], [2.0])


def test_jackknife_matches_delta_method_and_monte_carlo(o=trk):
    """Large-n behaviour fixed by the mathematics: var(R) ~ (var_s - 2 R cov_sg + R^2 var_g)/(n mu_g^2),
    and the spread of R over independent replications."""
    rng = np.random.default_rng(9)
    n, reps = 400, 300
    cov = np.array([[0.25, 0.3], [0.3, 4.0]])
    L = np.linalg.cholesky(cov)
    ratios, stderrs = [], []
    for _ in range(reps):
        z = rng.normal(size=(n, 2)) @ L.T + np.array([3.0, 6.0])
        r = o.offline_gns_sums(z[:, 0], z[:, 1])
        ratios.append(r["B_simple"])
        stderrs.append(r["stderr"])
    R = 2.0
    delta = np.sqrt((4.0 - 2 * R * 0.3 + R * R * 0.25) / n) / 3.0
    assert np.mean(stderrs) == pytest.approx(delta, rel=0.03)
    assert np.std(ratios, ddof=1) == pytest.approx(delta, rel=0.12)


def test_smaller_small_batch_gives_smaller_standard_error(o=trk):
    """The setting of Figure 2: true GNS = 1, the same number of examples processed; B_small = 1 has a
    lower jackknife standard error than B_small = 4 (each step's G2 and S from Eq. 4 and Eq. 5)."""
    import oracle
    rng = np.random.default_rng(10)
    D, B, steps = 64, 16, 300
    G = rng.normal(size=D)
    G /= np.linalg.norm(G)                                   # |G|^2 = 1 and tr(Sigma) = 1
    res = {}
    for b_small in (1, 4):
        g2s, ss = [], []
        for _ in range(steps):
            g = G + rng.normal(size=(B, D)) / np.sqrt(D)
            big = np.sum(g.mean(0) ** 2)
            small = np.mean(np.sum(g.reshape(B // b_small, b_small, D).mean(1) ** 2, axis=1))
            G2, S, _ = oracle.gns_from_norms(big, small, B, b_small)
            g2s.append(G2)
            ss.append(S)
        res[b_small] = o.offline_gns_sums(g2s, ss)
        assert res[b_small]["B_simple"] == pytest.approx(1.0, abs=5 * res[b_small]["stderr"])
    assert res[1]["stderr"] < res[4]["stderr"]


# ----------------------------------------------------------------------------- schedule
def test_schedule_hand_example_and_exact_ceiling(o=trk):
    g = GOLD["schedule"]
    got = [o.linear_accum_steps(t, g["ramp_tokens"], g["accum_final"]) for t in g["tokens"]]
    assert got == g["accum"]
    rng = np.random.default_rng(11)
    prev = 0
    for t in sorted(int(v) for v in rng.integers(0, 2 ** 62, 200)):
        a = o.linear_accum_steps(t, 2 ** 61 + 12345, 1000)
        want = min(1000, max(1, int(np.ceil(Fraction(1000 * t, 2 ** 61 + 12345)))))
        assert a == want and a >= prev
        prev = a
    assert o.linear_accum_steps(5, 0, 7) == 7


# ----------------------------------------------------------------------------- do these pins bite?
MUTATIONS = [
    ("alpha and 1-alpha swapped", "new[i, 0] = alpha * state[i, 0] + (1.0 - alpha) * g2[i]",
     "new[i, 0] = (1.0 - alpha) * state[i, 0] + alpha * g2[i]"),
    ("S smoothed from G2", "new[i, 1] = alpha * state[i, 1] + (1.0 - alpha) * s[i]",
     "new[i, 1] = alpha * state[i, 1] + (1.0 - alpha) * g2[i]"),
    ("no weight correction", "out[i, 0] = state[i, 0] / state[i, 2]", "out[i, 0] = state[i, 0]"),
    ("ratio inverted", "out[i, 2] = np.float64(state[i, 1]) / np.float64(state[i, 0])",
     "out[i, 2] = np.float64(state[i, 0]) / np.float64(state[i, 1])"),
    ("jackknife factor 1/n", "stderr = np.sqrt((n - 1.0) / n * np.sum((loo - rbar) ** 2))\n    return dict(mean_G2=float(np.mean(g2))",
     "stderr = np.sqrt(1.0 / n * np.sum((loo - rbar) ** 2))\n    return dict(mean_G2=float(np.mean(g2))"),
    ("deviation from the full ratio", "stderr = np.sqrt((n - 1.0) / n * np.sum((loo - rbar) ** 2))\n    return dict(mean_G2=float(np.mean(g2))",
     "stderr = np.sqrt((n - 1.0) / n * np.sum((loo - ratio) ** 2))\n    return dict(mean_G2=float(np.mean(g2))"),
    ("mean of ratios", "ratio = np.mean(s) / np.mean(g2)", "ratio = np.mean(s / g2)"),
    ("sums form: element not removed from the denominator", "loo = (sum_s - s) / (sum_g - g2)",
     "loo = (sum_s - s) / (sum_g - sum_g / n)"),
    ("bias correction sign", "B_simple_jack=float(n * ratio - (n - 1.0) * rbar))\n\n\ndef offline_gns_sums",
     "B_simple_jack=float(n * ratio + (n - 1.0) * rbar))\n\n\ndef offline_gns_sums"),
    ("schedule floors", "a = -((-accum_final * tokens_seen) // ramp_tokens)",
     "a = (accum_final * tokens_seen) // ramp_tokens"),
]


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_fails_some_pin(name, old, new):
    text = open(trk.__file__).read()
    assert text.count(old) == 1, f"mutation target not found exactly once: {old!r}"
    mod = types.ModuleType("mutated_tracker")
    mod.__file__ = trk.__file__
    exec(compile(text.replace(old, new), "mutated_tracker", "exec"), mod.__dict__)
    pins = [test_ema_hand_example, test_ema_constant_sequence_is_reproduced_at_every_step,
            lambda o: test_ema_equals_geometric_weighted_mean(0.3, o), test_ema_limits,
            test_jackknife_hand_example, test_jackknife_of_a_plain_mean_is_the_textbook_standard_error,
            test_jackknife_two_forms_agree_and_symmetries, test_schedule_hand_example_and_exact_ceiling]
    caught = 0
    for pin in pins:
        try:
            pin(o=mod) if not isinstance(pin, types.LambdaType) or pin.__name__ != "<lambda>" else pin(mod)
        except (AssertionError, ValueError, ZeroDivisionError):
            caught += 1
    assert caught >= 1, f"no pin noticed: {name}"
