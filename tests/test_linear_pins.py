"""Pins for oracle/linear_pegn_oracle.py (Section 3, Algorithm 1): a hand-worked example, brute-force
loops, the two closed forms the paper quotes for per-example norms (Section 2.2: the two-dimensional
product form and the three-dimensional Gram form), a library's autograd on one example at a time,
and symmetries.  The last test plants mistakes in a copy of the oracle."""
import json
import os
import types

import numpy as np
import pytest

from oracle import linear_pegn_oracle as lin

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "linear_pegn_hand_example.json")))


def _rand(B, T, K, L, seed=0):
    rng = np.random.default_rng(seed)
    return rng.normal(size=(B, T, K)), rng.normal(size=(B, T, L))


def test_hand_example(o=lin):
    r = o.linear_pegn(GOLD["x"], GOLD["g"], want_pe=True)
    np.testing.assert_array_equal(r["pe"], np.array(GOLD["expected"]["pe"], dtype=np.float64))
    np.testing.assert_array_equal(r["s"], GOLD["expected"]["s"])
    np.testing.assert_array_equal(r["w"], GOLD["expected"]["w"])


def test_brute_force_loops(o=lin):
    x, g = _rand(3, 4, 5, 2, seed=1)
    r = o.linear_pegn(x, g, want_pe=True)
    for b in range(3):
        tot = 0.0
        for k in range(5):
            for l in range(2):
                acc = 0.0
                for t in range(4):
                    acc += x[b, t, k] * g[b, t, l]
                assert r["pe"][b, k, l] == pytest.approx(acc, rel=1e-13, abs=1e-15)
                tot += acc * acc
        assert r["s"][b] == pytest.approx(tot, rel=1e-13)
    np.testing.assert_allclose(r["w"], r["pe"].sum(0), rtol=1e-13, atol=1e-14)


def test_T1_product_form(o=lin):
    """Section 2.2, two-dimensional case: n_b^2 = (sum_i x_bi^2) * (sum_k g_bk^2)."""
    x, g = _rand(6, 1, 7, 9, seed=2)
    r = o.linear_pegn(x, g)
    np.testing.assert_allclose(r["s"], (x[:, 0] ** 2).sum(1) * (g[:, 0] ** 2).sum(1), rtol=1e-13)


def test_gram_form(o=lin):
    """Section 2.2, three-dimensional case: n_b^2 = <X_b X_b^T, G_b G_b^T>_F (O(T^2) memory)."""
    x, g = _rand(4, 6, 5, 3, seed=3)
    r = o.linear_pegn(x, g)
    for b in range(4):
        assert r["s"][b] == pytest.approx(np.sum((x[b] @ x[b].T) * (g[b] @ g[b].T)), rel=1e-12)


def test_sampled_entries_and_gram_form_agree_with_the_full_definition(o=lin):
    """The two helpers used where the full result is out of reach are pinned to the definition here."""
    x, g = _rand(3, 9, 6, 5, seed=11)
    r = o.linear_pegn(x, g)
    ks, ls = [0, 5, 2, 3], [4, 0, 2, 1]
    np.testing.assert_allclose(o.linear_pegn_entries(x, g, ks, ls), r["w"][ks, ls], rtol=1e-12, atol=1e-13)
    for b in range(3):
        assert o.gram_sq_norm(x[b], g[b]) == pytest.approx(r["s"][b], rel=1e-12)


def test_weight_gradient_is_the_flattened_contraction(o=lin):
    x, g = _rand(3, 5, 4, 6, seed=4)
    r = o.linear_pegn(x, g)
    np.testing.assert_allclose(r["w"], np.einsum("btk,btl->kl", x, g), rtol=1e-12, atol=1e-13)


def test_library_autograd_one_example_at_a_time(o=lin):
    """y = x W^T with W [L,K]; for loss = sum(y * c) the gradient of W for example b alone is w_b^T."""
    import torch
    x, g = _rand(3, 5, 4, 6, seed=5)
    r = o.linear_pegn(x, g, want_pe=True)
    W = torch.zeros((6, 4), dtype=torch.float64, requires_grad=True)
    for b in range(3):
        y = torch.nn.functional.linear(torch.from_numpy(x[b]), W)
        (grad,) = torch.autograd.grad((y * torch.from_numpy(g[b])).sum(), W)
        np.testing.assert_allclose(r["pe"][b], grad.numpy().T, rtol=1e-12, atol=1e-13)
        assert r["s"][b] == pytest.approx(float((grad ** 2).sum()), rel=1e-12)


def test_symmetries(o=lin):
    x, g = _rand(3, 5, 4, 6, seed=6)
    r = o.linear_pegn(x, g)
    # scaling x by a and g by c scales w by a*c and s by (a*c)^2
    r2 = o.linear_pegn(3.0 * x, -0.5 * g)
    np.testing.assert_allclose(r2["w"], -1.5 * r["w"], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(r2["s"], 2.25 * r["s"], rtol=1e-13)
    # permuting the positions t of one example changes nothing; permuting examples permutes s
    perm = np.random.default_rng(7).permutation(5)
    r3 = o.linear_pegn(x[:, perm], g[:, perm])
    np.testing.assert_allclose(r3["s"], r["s"], rtol=1e-12)
    r4 = o.linear_pegn(x[::-1], g[::-1])
    np.testing.assert_allclose(r4["s"], r["s"][::-1], rtol=1e-13)
    np.testing.assert_allclose(r4["w"], r["w"], rtol=1e-12, atol=1e-13)
    # swapping the roles of x and g transposes w and keeps s
    r5 = o.linear_pegn(g, x)
    np.testing.assert_allclose(r5["w"], r["w"].T, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(r5["s"], r["s"], rtol=1e-13)
    # B = 1: the per-example norm is the norm of the weight gradient
    r6 = o.linear_pegn(x[:1], g[:1])
    assert r6["s"][0] == pytest.approx(np.sum(r6["w"] ** 2), rel=1e-13)
    # identical examples: w = B * w_0, s all equal
    r7 = o.linear_pegn(np.repeat(x[:1], 4, 0), np.repeat(g[:1], 4, 0))
    np.testing.assert_allclose(r7["w"], 4 * r6["w"], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(r7["s"], r6["s"][0], rtol=1e-13)
    with pytest.raises(ValueError):
        o.linear_pegn(x, g[:, :4])


MUTATIONS = [
    ("positions mispaired (x reversed along t)", "w_b = x[b].T @ g[b]", "w_b = x[b].T[:, ::-1] @ g[b]"),
    ("x not transposed (outer sum of rows)", "w_b = x[b].T @ g[b]", "w_b = np.outer(x[b].sum(0), g[b].sum(0))"),
    ("norm is a sum of abs", "s[b] = np.sum(w_b * w_b)", "s[b] = np.sum(np.abs(w_b))"),
    ("norm of the running total", "s[b] = np.sum(w_b * w_b)", "s[b] = np.sum((w + w_b) * (w + w_b))"),
    ("mean over b in the weight gradient", "        w += w_b\n", "        w += w_b / B\n"),
    ("square root taken", "s[b] = np.sum(w_b * w_b)", "s[b] = np.sqrt(np.sum(w_b * w_b))"),
]


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_fails_some_pin(name, old, new):
    text = open(lin.__file__).read()
    assert text.count(old) == 1, f"mutation target not found exactly once: {old!r}"
    mod = types.ModuleType("mutated_linear")
    exec(compile(text.replace(old, new), "mutated_linear", "exec"), mod.__dict__)
    caught = 0
    for pin in (test_hand_example, test_brute_force_loops, test_T1_product_form, test_gram_form,
                test_weight_gradient_is_the_flattened_contraction, test_symmetries):
        try:
            pin(o=mod)
        except (AssertionError, ValueError):
            caught += 1
    assert caught >= 1, f"no pin noticed: {name}"
