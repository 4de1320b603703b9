"""Pins for oracle/embedding_pegn_oracle.py (Appendix B, embedding-layer algorithm): a hand-worked
example, brute-force loops, closed forms for the two extreme id patterns, a library's autograd on one
example at a time, symmetries; the last test plants mistakes in a copy of the oracle."""
import json
import os
import types

import numpy as np
import pytest

from oracle import embedding_pegn_oracle as emb

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "embedding_pegn_hand_example.json")))


def _rand(B, T, D, V, seed=0):
    rng = np.random.default_rng(seed)
    return rng.integers(0, V, (B, T)), rng.normal(size=(B, T, D))


def test_hand_example(o=emb):
    r = o.embedding_pegn(np.array(GOLD["ids"]), GOLD["g"], GOLD["V"], want_pe=True)
    np.testing.assert_array_equal(r["pe"], np.array(GOLD["expected"]["pe"], dtype=np.float64))
    np.testing.assert_array_equal(r["s"], GOLD["expected"]["s"])
    np.testing.assert_array_equal(r["w"], GOLD["expected"]["w"])


def test_brute_force_loops(o=emb):
    ids, g = _rand(3, 7, 4, 5, seed=1)
    r = o.embedding_pegn(ids, g, 5, want_pe=True)
    for b in range(3):
        tot = 0.0
        for v in range(5):
            for d in range(4):
                acc = 0.0
                for t in range(7):
                    if ids[b, t] == v:
                        acc += g[b, t, d]
                assert r["pe"][b, v, d] == pytest.approx(acc, rel=1e-13, abs=1e-15)
                tot += acc * acc
        assert r["s"][b] == pytest.approx(tot, rel=1e-13)
    np.testing.assert_allclose(r["w"], r["pe"].sum(0), rtol=1e-13, atol=1e-14)


def test_all_ids_distinct_and_all_ids_equal(o=emb):
    """Distinct ids within an example: nothing is summed before squaring, s_b = sum_t |g_bt|^2.
    One id throughout: everything is, s_b = |sum_t g_bt|^2 (the LayerNorm-bias form)."""
    rng = np.random.default_rng(2)
    g = rng.normal(size=(4, 6, 5))
    ids = np.stack([rng.permutation(9)[:6] for _ in range(4)])
    np.testing.assert_allclose(o.embedding_pegn(ids, g, 9)["s"], (g ** 2).sum((1, 2)), rtol=1e-13)
    same = np.full((4, 6), 3)
    r = o.embedding_pegn(same, g, 9)
    np.testing.assert_allclose(r["s"], (g.sum(1) ** 2).sum(1), rtol=1e-13)
    assert np.count_nonzero(np.abs(r["w"]).sum(1)) == 1


def test_library_autograd_one_example_at_a_time(o=emb):
    import torch
    ids, g = _rand(3, 8, 4, 6, seed=3)
    r = o.embedding_pegn(ids, g, 6, want_pe=True)
    W = torch.zeros((6, 4), dtype=torch.float64, requires_grad=True)
    total = torch.zeros_like(W)
    for b in range(3):
        y = torch.nn.functional.embedding(torch.from_numpy(ids[b]), W)
        (grad,) = torch.autograd.grad((y * torch.from_numpy(g[b])).sum(), W)
        np.testing.assert_allclose(r["pe"][b], grad.numpy(), rtol=1e-13, atol=1e-14)
        assert r["s"][b] == pytest.approx(float((grad ** 2).sum()), rel=1e-13)
        total += grad
    np.testing.assert_allclose(r["w"], total.numpy(), rtol=1e-13, atol=1e-14)


def test_symmetries(o=emb):
    ids, g = _rand(3, 8, 4, 6, seed=4)
    r = o.embedding_pegn(ids, g, 6)
    perm = np.random.default_rng(5).permutation(8)                 # order of positions is irrelevant
    r2 = o.embedding_pegn(ids[:, perm], g[:, perm], 6)
    np.testing.assert_allclose(r2["s"], r["s"], rtol=1e-12)
    np.testing.assert_allclose(r2["w"], r["w"], rtol=1e-12, atol=1e-13)
    relabel = np.random.default_rng(6).permutation(6)              # renaming ids permutes rows of w, keeps s
    r3 = o.embedding_pegn(relabel[ids], g, 6)
    np.testing.assert_allclose(r3["s"], r["s"], rtol=1e-13)
    np.testing.assert_allclose(r3["w"][relabel], r["w"], rtol=1e-13)
    r4 = o.embedding_pegn(ids, -2.0 * g, 6)                        # scale
    np.testing.assert_allclose(r4["s"], 4.0 * r["s"], rtol=1e-13)
    r5 = o.embedding_pegn(ids, g, 10)                              # a larger vocabulary adds empty rows only
    np.testing.assert_allclose(r5["w"][:6], r["w"], rtol=1e-13)
    assert not r5["w"][6:].any()
    for bad in (np.array([[6]]), np.array([[-1]])):
        with pytest.raises(ValueError):
            o.embedding_pegn(bad, np.zeros((1, 1, 2)), 6)


MUTATIONS = [
    ("norm of rows summed without grouping by id", "s[b] = np.sum(w_b * w_b)", "s[b] = np.sum(g[b] * g[b])"),
    ("everything summed before squaring", "s[b] = np.sum(w_b * w_b)", "s[b] = np.sum(g[b].sum(0) ** 2)"),
    ("row index off by one", "w_b[int(ids[b, t])] += g[b, t]", "w_b[(int(ids[b, t]) + 1) % V] += g[b, t]"),
    ("ids of example 0 used for all", "w_b[int(ids[b, t])] += g[b, t]", "w_b[int(ids[0, t])] += g[b, t]"),
    ("mean over b in the weight gradient", "        w += w_b\n", "        w += w_b / B\n"),
    ("a repeated id overwrites instead of adding", "w_b[int(ids[b, t])] += g[b, t]", "w_b[int(ids[b, t])] = g[b, t]"),
    ("per-example gradient not cleared between examples", "w_b = np.zeros((V, D))                       # example",
     "w_b = w if b else np.zeros((V, D))           # example"),
]


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_fails_some_pin(name, old, new):
    text = open(emb.__file__).read()
    assert text.count(old) == 1, f"mutation target not found exactly once: {old!r}"
    mod = types.ModuleType("mutated_embedding")
    exec(compile(text.replace(old, new), "mutated_embedding", "exec"), mod.__dict__)
    caught = 0
    for pin in (test_hand_example, test_brute_force_loops, test_all_ids_distinct_and_all_ids_equal, test_symmetries):
        try:
            pin(o=mod)
        except (AssertionError, ValueError):
            caught += 1
    assert caught >= 1, f"no pin noticed: {name}"
