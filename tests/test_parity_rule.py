"""The comparison rule of the GPU parity tests, checked on the CPU against planted errors.

The reference is the oracle's dx; the "device output" is made here from it: correctly rounded
(must pass), or with a planted error (must fail, and by the criterion named).  No GPU code runs.
"""
import numpy as np
import pytest

import oracle
import parity_util as pu
from paper_2411_00999_amd import workloads


def _ref_dx(cfg, B, T, D):
    inp = workloads.make_inputs(cfg, B=B, T=T, D=D)
    ref = oracle.ln_bwd_pegn(inp.x, inp.dy, inp.gamma, inp.eps, want_pe=False)
    return inp, ref["dx"].reshape(-1, D)


CASES = [(1, 4, 128, 256), (2, 2, 64, 768), (3, 2, 64, 2048), (4, 8, 16, 1024), (5, 2, 8, 8192), (1, 2, 3, 1),
         (2, 1, 1, 8), (1, 2, 5, 2)]


@pytest.mark.parametrize("cfg,B,T,D", CASES)
def test_correctly_rounded_output_passes(cfg, B, T, D):
    inp, dx = _ref_dx(cfg, B, T, D)
    bf = inp.dtype == "bf16"
    out = pu.rne_bf16(dx) if bf else dx.astype(np.float32).astype(np.float64)
    pu.check_close("dx", out, dx, pu.TOL_BF16 if bf else pu.TOL_F32, bf16_output=bf,
                   floor_rms=pu.dx_term_rms(inp))


def test_rne_bf16_is_round_to_nearest_even():
    rng = np.random.default_rng(5)
    v = rng.standard_normal(4096) * np.exp(rng.uniform(-20, 20, 4096))
    got = pu.rne_bf16(v)
    want = workloads.round_to_bf16(v.astype(np.float32)).astype(np.float64)   # the generator's own rounding
    # float64 -> float32 first can move a value across a bf16 tie only for a handful in 2^29; none here
    np.testing.assert_array_equal(got, want)
    assert pu.rne_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0              # tie -> even (down)
    assert pu.rne_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6   # tie -> even (up)


@pytest.mark.parametrize("cfg,B,T,D", [(1, 4, 128, 256), (3, 2, 64, 2048), (4, 8, 16, 1024)])
def test_thinly_spread_error_is_caught_by_the_l2_criterion(cfg, B, T, D):
    """An error of 0.9 x the elementwise bound on every element passes criterion (2) by
    construction; criterion (1) must be the one that rejects it -- for dx too, whose rms sits a
    hair below its floor."""
    inp, dx = _ref_dx(cfg, B, T, D)
    bf = inp.dtype == "bf16"
    tol = pu.TOL_BF16 if bf else pu.TOL_F32
    floor = pu.dx_term_rms(inp)
    rms = np.linalg.norm(dx) / np.sqrt(dx.size)
    assert rms < floor                       # the situation in which the L2 check used to be skipped
    sign = np.where(np.random.default_rng(1).random(dx.shape) < 0.5, -1.0, 1.0)
    bound = tol * (np.abs(dx) + floor) + (pu.bf16_half_ulp(dx) if bf else 0.0)
    out = dx + 0.9 * sign * bound
    with pytest.raises(AssertionError, match="L2 relative error"):
        pu.check_close("dx", out, dx, tol, bf16_output=bf, floor_rms=floor)


@pytest.mark.parametrize("cfg,B,T,D", [(2, 2, 64, 768), (3, 2, 64, 2048)])
def test_one_percent_scale_error_is_caught(cfg, B, T, D):
    """The realistic failure: every element off by a constant factor (Appendix D.3 tells of one)."""
    inp, dx = _ref_dx(cfg, B, T, D)
    out = pu.rne_bf16(dx * 1.01)
    with pytest.raises(AssertionError):
        pu.check_close("dx", out, dx, pu.TOL_BF16, bf16_output=True, floor_rms=pu.dx_term_rms(inp))
    # and the L2 criterion alone rejects it: ||1% of ref|| is five times tol
    rel = np.linalg.norm(out - dx) / np.linalg.norm(dx)
    q = np.linalg.norm(pu.rne_bf16(dx) - dx) / np.linalg.norm(dx)
    assert rel > max(pu.TOL_BF16, q + pu.BF16_L2_SLACK)


def test_single_bad_element_is_caught_by_the_elementwise_criterion():
    inp, dx = _ref_dx(1, 4, 128, 256)
    out = dx.copy()
    out[7, 3] += 50 * pu.TOL_F32 * pu.dx_term_rms(inp)     # invisible in the L2 norm of 131072 elements
    with pytest.raises(AssertionError, match=r"\|out-ref\|"):
        pu.check_close("dx", out, dx, pu.TOL_F32, floor_rms=pu.dx_term_rms(inp))


def test_fully_cancelling_dx_is_compared_against_the_floor():
    """D = 1: dx is exactly zero; the L2 check runs against floor_rms*sqrt(size), not skipped."""
    inp, dx = _ref_dx(1, 2, 3, 1)
    assert np.all(dx == 0.0)
    floor = pu.dx_term_rms(inp)
    pu.check_close("dx", np.full_like(dx, 0.5 * pu.TOL_F32 * floor), dx, pu.TOL_F32, floor_rms=floor)
    with pytest.raises(AssertionError):
        pu.check_close("dx", np.full_like(dx, 3.0 * pu.TOL_F32 * floor), dx, pu.TOL_F32, floor_rms=floor)
