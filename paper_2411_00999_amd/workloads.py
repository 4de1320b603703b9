"""Seeded synthetic inputs for the LayerNorm-backward + per-example-norm path.

This module only draws numbers.  It holds none of the method's arithmetic, is
imported by the tests, the benchmark and the smoke check, and serves both the
CPU oracle and the HIP library with the *same* values: every array returned is
float32 and, for the bf16 workloads, already rounded to a bf16-representable
value (round to nearest even), so both sides start from identical inputs.

The five workloads stand in for the paper's language-model LayerNorm shapes
(111M GPT with hidden 768; 1.3B GPT-2-like model; bf16 mixed precision or
fp32 -- Section 4 and Appendix D.3).  No dataset is involved on this path.
The second argument of N(.,.) below is a standard deviation.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

BASE_SEED = 241100999

#          B     T     D   dtype   layers
SHAPES = {
    1: (4, 128, 256, "f32", 1),
    2: (8, 1024, 768, "bf16", 1),
    3: (16, 2048, 2048, "bf16", 48),
    4: (512, 64, 1024, "bf16", 1),
    5: (8, 4096, 8192, "bf16", 1),
}
EPS = 1e-5


@dataclass
class LNInputs:
    config: int
    layer: int
    B: int
    T: int
    D: int
    dtype: str          # "f32" or "bf16": storage type of x, dy, dx on the device
    eps: float
    x: np.ndarray       # [B,T,D] float32 (bf16-representable when dtype == "bf16")
    dy: np.ndarray      # [B,T,D] float32 (same)
    gamma: np.ndarray   # [D] float32 (same)
    beta: np.ndarray    # [D] float32 (same); never enters the backward

    @property
    def rows(self) -> int:
        return self.B * self.T

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    @property
    def algorithmic_bytes(self) -> int:
        """read x + read dy + write dx."""
        return 3 * self.B * self.T * self.D * self.elem_bytes


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """float32 -> nearest bf16 (ties to even), returned as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    out = ((u + r) & np.uint32(0xFFFF0000)).view(np.float32)
    return np.where(np.isfinite(a), out, a).astype(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """Upper 16 bits of bf16-representable float32 values, as uint16."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    if np.any(u & np.uint32(0xFFFF)):
        raise ValueError("values are not bf16-representable")
    return (u >> np.uint32(16)).astype(np.uint16)


def bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """uint16 bf16 patterns -> float32 (exact)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def seed_for(config: int, layer: int = 0) -> int:
    return BASE_SEED + 1000 * config + layer


def _normal(rng, shape, std=1.0):
    out = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        out *= np.float32(std)
    return out


def make_inputs(config: int, layer: int = 0, B: Optional[int] = None, T: Optional[int] = None,
                D: Optional[int] = None, dtype: Optional[str] = None,
                signal: float = 0.0) -> LNInputs:
    """Inputs of workload ``config`` (1..5), optionally at a reduced shape.

    ``signal`` > 0 adds to dy a fixed [T,D] pattern of that standard deviation
    shared by every example, so that the true gradient is not zero and the
    noise-scale ratio is well conditioned.
    """
    if config not in SHAPES:
        raise ValueError(f"unknown workload {config}")
    B0, T0, D0, dt0, _ = SHAPES[config]
    B, T, D = B or B0, T or T0, D or D0
    dtype = dtype or dt0
    rng = np.random.default_rng(seed_for(config, layer))
    shape = (B, T, D)

    if config == 1:
        x = _normal(rng, shape)
        dy = _normal(rng, shape, 1e-2)
        gamma = 1.0 + _normal(rng, (D,), 0.1)
        beta = _normal(rng, (D,), 0.1)
    elif config == 2:
        x = _normal(rng, shape)
        dy = _normal(rng, shape, 1e-3)
        gamma = 1.0 + _normal(rng, (D,), 0.05)
        beta = _normal(rng, (D,), 0.1)
    elif config == 3:
        scale = np.exp(_normal(rng, (B, T, 1), 0.5)).astype(np.float32)   # LogNormal(0, 0.5) per row
        x = _normal(rng, shape)
        x *= scale
        dy = _normal(rng, shape, 1e-3)
        gamma = 1.0 + _normal(rng, (D,), 0.05)
        beta = _normal(rng, (D,), 0.1)
    elif config == 4:
        x = _normal(rng, shape)
        dy = _normal(rng, shape, 1e-3)
        half = B // 2
        if half > 1:                      # examples 0..half-1 are copies of example 0
            x[1:half] = x[0]
            dy[1:half] = dy[0]
        gamma = 1.0 + _normal(rng, (D,), 0.05)
        beta = _normal(rng, (D,), 0.1)
    else:  # config 5
        x = np.empty(shape, dtype=np.float32)
        dy = np.empty(shape, dtype=np.float32)
        n_out = max(1, int(round(0.01 * D)))
        chans = np.sort(rng.choice(D, size=n_out, replace=False))
        for b in range(B):               # per example: bounds the float64 temporaries
            xb = _normal(rng, (T, D))
            xb[:, chans] *= np.float32(20.0)
            x[b] = xb
            dy[b] = (rng.standard_t(3.0, size=(T, D)) * 1e-3).astype(np.float32)
        gamma = 1.0 + _normal(rng, (D,), 0.05)
        beta = _normal(rng, (D,), 0.1)

    if signal > 0.0:
        m = _normal(np.random.default_rng(seed_for(config, layer) + 500), (T, D), signal)
        dy += m[None]

    gamma = gamma.astype(np.float32)
    beta = beta.astype(np.float32)
    if dtype == "bf16":
        x, dy, gamma, beta = (round_to_bf16(a) for a in (x, dy, gamma, beta))
    elif dtype != "f32":
        raise ValueError(f"unknown dtype {dtype}")
    return LNInputs(config, layer, B, T, D, dtype, EPS, x, dy, gamma, beta)


# ----------------------------------------------------------------------------- linear layers
# Shapes of the linear layers next to the LayerNorm workloads: (B, T, K, L).  "gpt111m" are the four
# projections of a block with hidden size 768 (Section 4), "gpt1p3b" the MLP up-projection of the
# hidden-2048 model of Section 5.2; inputs are what such a layer sees: unit-variance activations
# after a LayerNorm and small zero-mean output gradients.
LINEAR_SHAPES = {
    "gpt111m_qkv": (8, 1024, 768, 2304),
    "gpt111m_proj": (8, 1024, 768, 768),
    "gpt111m_up": (8, 1024, 768, 3072),
    "gpt111m_down": (8, 1024, 3072, 768),
    "gpt1p3b_up": (16, 2048, 2048, 8192),
}


def make_linear_inputs(seed: int, B: int, T: int, K: int, L: int, dtype: str = "bf16", signal: float = 0.0):
    """(x [B,T,K], g [B,T,L]) float32 arrays (already rounded to bf16 values when dtype is "bf16").
    ``signal`` > 0 adds to g a fixed [T,L] pattern shared by every example."""
    rng = np.random.default_rng(BASE_SEED + 500_000 + seed)
    x = _normal(rng, (B, T, K))
    g = _normal(rng, (B, T, L), 1e-3)
    if signal > 0.0:
        g += _normal(rng, (1, T, L), signal)
    if dtype == "bf16":
        x, g = round_to_bf16(x), round_to_bf16(g)
    return x, g


# ----------------------------------------------------------------------------- embedding layer
# The token embedding of the paper's GPT models: vocabulary 50257, hidden 768 (Section 4) or 2048
# (Section 5.2).  Ids follow a Zipf law over a randomly ordered vocabulary, which is what text looks
# like to this layer: a few ids many times per example, most ids never.
EMBEDDING_SHAPES = {
    "gpt111m_wte": (8, 1024, 768, 50257),
    "gpt1p3b_wte": (16, 2048, 2048, 50257),
}


def make_embedding_inputs(seed: int, B: int, T: int, D: int, V: int, dtype: str = "bf16", zipf_a: float = 1.2):
    """(ids [B,T] int64 in [0,V), g [B,T,D] float32 (rounded to bf16 values when dtype is "bf16"))."""
    rng = np.random.default_rng(BASE_SEED + 700_000 + seed)
    order = rng.permutation(V)
    ids = order[(rng.zipf(zipf_a, size=(B, T)) - 1) % V].astype(np.int64)
    g = _normal(rng, (B, T, D), 1e-3)
    if dtype == "bf16":
        g = round_to_bf16(g)
    return ids, g


# ------------------------------------------------------------------ host <-> device plumbing
def to_device(arr32: np.ndarray, dtype: str):
    """float32 host values -> device tensor of the workload's storage type (exact)."""
    import torch
    if dtype == "bf16":
        bits = bf16_bits(arr32)
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(arr32, dtype=np.float32)).cuda()


def to_host64(t) -> np.ndarray:
    """device tensor (fp32 or bf16) -> float64 numpy (exact)."""
    import torch
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy().astype(np.float64)
    return t.cpu().numpy().astype(np.float64)


def make_inputs_device(config: int, set_index: int = 0, dtype: Optional[str] = None):
    """Workload ``config`` at full size drawn ON the GPU (torch generator, seeded by workload and set index):
    (x, dy, gamma) device tensors with the workload's distributions.  For timing legs that rotate over many
    buffer sets, where drawing gigabytes on the host would take longer than the measurement; the parity tests
    use make_inputs, whose values the oracle reads too."""
    import torch
    B, T, D, dt0, _ = SHAPES[config]
    dtype = dtype or dt0
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed_for(config, 0) * 4096 + set_index)

    def normal(shape, std=1.0):
        return torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32) * std

    x = normal((B, T, D))
    if config == 3:
        x *= torch.exp(normal((B, T, 1), 0.5))
    if config == 5:
        n_out = max(1, int(round(0.01 * D)))
        chans = torch.randperm(D, generator=gen, device="cuda")[:n_out]
        x[:, :, chans] *= 20.0
    x = x.to(tdt)
    if config == 5:                       # Student-t(3) = normal / sqrt(chi2_3 / 3), example by example
        dy = torch.empty((B, T, D), dtype=tdt, device="cuda")
        for b in range(B):
            chi2 = sum(normal((T, D)) ** 2 for _ in range(3))
            dy[b] = (normal((T, D)) / torch.sqrt(chi2 / 3.0) * 1e-3).to(tdt)
    else:
        dy = normal((B, T, D), 1e-2 if config == 1 else 1e-3).to(tdt)
    if config == 4 and B // 2 > 1:
        x[1:B // 2] = x[0]
        dy[1:B // 2] = dy[0]
    gamma = (1.0 + normal((D,), 0.1 if config == 1 else 0.05)).to(tdt)
    return x, dy, gamma
