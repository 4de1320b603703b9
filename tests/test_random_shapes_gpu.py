"""Seeded random shapes through every path, each compared with its oracle: a net for the cases nobody thought of
(ragged widths, one-row examples, tiles that end mid-way, ids that are all alike or all different)."""
import numpy as np
import pytest

from paper_2411_00999_amd import workloads
import parity_util as pu
import test_parity_gpu as tp

pytestmark = pytest.mark.gpu

SEED = workloads.BASE_SEED + 7_000_000


def _shapes(n, seed, draw):
    rng = np.random.default_rng(SEED + seed)
    return [draw(rng) for _ in range(n)]


LN_SHAPES = _shapes(24, 1, lambda r: (int(r.integers(1, 7)), int(r.integers(1, 41)),
                                       int(r.choice([r.integers(1, 700), 8 * r.integers(1, 140), 64 * r.integers(1, 40)])),
                                       str(r.choice(["bf16", "f32"]))))


@pytest.mark.parametrize("B,T,D,dtype", LN_SHAPES)
def test_layernorm_random_shapes(B, T, D, dtype):
    inp = workloads.make_inputs(1, B=B, T=T, D=D, dtype=dtype, signal=1e-2)
    ref = tp._oracle(inp)
    for saved in (False, True):
        pu.compare_with_oracle(inp, pu.run_gpu(inp, saved_stats=saved), ref)
    pu.compare_with_oracle(inp, pu.run_gpu(inp, pegn=False), ref, pegn=False)


LIN_SHAPES = _shapes(16, 2, lambda r: (int(r.integers(1, 6)), int(r.integers(1, 200)),
                                        int(r.choice([8 * r.integers(1, 80), r.integers(1, 300)])),
                                        int(r.choice([8 * r.integers(1, 60), r.integers(1, 200)])),
                                        str(r.choice(["bf16", "f32"]))))


@pytest.mark.parametrize("B,T,K,L,dtype", LIN_SHAPES)
def test_linear_random_shapes(B, T, K, L, dtype):
    x, g = workloads.make_linear_inputs(B * 1000 + T, B, T, K, L, dtype, signal=1e-3)
    tp._check_linear(x, g, tp._run_linear(x, g, dtype))
    w0 = np.random.default_rng(SEED + K * L).normal(0, 1e-2, (K, L))
    tp._check_linear(x, g, tp._run_linear(x, g, dtype, w0=w0), w0=w0)


EMB_SHAPES = _shapes(16, 3, lambda r: (int(r.integers(1, 9)), int(r.integers(1, 160)),
                                        int(r.choice([8 * r.integers(1, 100), r.integers(1, 300)])),
                                        int(r.choice([1, 2, 5, 40, 700, 50257])), str(r.choice(["bf16", "f32"]))))


@pytest.mark.parametrize("B,T,D,V,dtype", EMB_SHAPES)
def test_embedding_random_shapes(B, T, D, V, dtype):
    ids, g = workloads.make_embedding_inputs(B * 1000 + T, B, T, D, V, dtype)
    tp._check_embedding(ids, g, V, tp._run_embedding(ids, g, V, dtype))
    rng = np.random.default_rng(SEED + D + V)
    uniform = rng.integers(0, V, (B, T))            # few repeats when V is large, all alike when V is 1
    tp._check_embedding(uniform, g, V, tp._run_embedding(uniform, g, V, dtype, int32=True))
