"""Do the pins bite?  Each case plants ONE plausible mistake in a copy of the oracle's C source
(on the CPU, in a temporary directory), loads the mutated library in place of the real one and
re-runs the pin tests: at least one of them has to fail.  A mutation that every pin lets through
would mean the oracle could carry that mistake unnoticed."""
import ctypes
import os
import subprocess

import pytest

import oracle
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "ln_pegn_oracle.c")

# (name, text in the oracle source, replacement)
MUTATIONS = [
    ("unbiased variance", "const double var = ss / (double)D;", "const double var = ss / (double)(D - 1);"),
    ("eps outside the root", "*rstd = 1.0 / sqrt(var + eps);", "*rstd = 1.0 / (sqrt(var) + eps);"),
    ("mean over D-1", "const double mu = sum / (double)D;", "const double mu = sum / (double)(D - 1);"),
    ("dx: mean(dyh) term dropped", "dx[t * D + k] = rstd * (dyh - c2 - xhat * c1);",
     "dx[t * D + k] = rstd * (dyh - xhat * c1);"),
    ("dx: projection term sign", "dx[t * D + k] = rstd * (dyh - c2 - xhat * c1);",
     "dx[t * D + k] = rstd * (dyh - c2 + xhat * c1);"),
    ("dx: rstd factor dropped", "dx[t * D + k] = rstd * (dyh - c2 - xhat * c1);",
     "dx[t * D + k] = (dyh - c2 - xhat * c1);"),
    ("dx: c1 is a sum, not a mean", "const double c1 = sum_dyh_xhat / (double)D;",
     "const double c1 = sum_dyh_xhat;"),
    ("dx: gamma forgotten", "const double dyh = gr[k] * gamma[k];\n                dx[t * D + k]",
     "const double dyh = gr[k];\n                dx[t * D + k]"),
    ("gamma grad from x, not xhat", "g_gamma[k] += gr[k] * xhat;", "g_gamma[k] += gr[k] * xr[k];"),
    ("gamma grad from dy*gamma", "g_gamma[k] += gr[k] * xhat;", "g_gamma[k] += dyh * xhat;"),
    ("beta grad from dy*gamma", "g_beta[k] += gr[k];", "g_beta[k] += dyh;"),
    ("norm is a sum of abs", "sg += gg[b * D + k] * gg[b * D + k];", "sg += fabs(gg[b * D + k]);"),
    ("beta norm taken from gamma grads", "sb += gb[b * D + k] * gb[b * D + k];",
     "sb += gg[b * D + k] * gg[b * D + k];"),
    ("batch grad is a mean over b", "dgamma[k] = a;", "dgamma[k] = a / (double)B;"),
    ("B^2 correction applied once", "small += mean_s * pe_scale * pe_scale;", "small += mean_s * pe_scale;"),
    ("sum over b instead of mean", "mean_s /= (double)B;", "mean_s /= 1.0;"),
    ("Eq. 4 norms swapped", "(b_big * g_big_sq - b_small * g_small_sq)", "(b_big * g_small_sq - b_small * g_big_sq)"),
    ("Eq. 4 batch sizes swapped", "(b_big * g_big_sq - b_small * g_small_sq)", "(b_small * g_big_sq - b_big * g_small_sq)"),
    ("Eq. 5 denominator sign", "(1.0 / b_small - 1.0 / b_big)", "(1.0 / b_big - 1.0 / b_small)"),
    ("Eq. 5 without reciprocals", "(1.0 / b_small - 1.0 / b_big)", "(b_big - b_small)"),
    ("Eq. 3 inverted", "out[2] = S / G2;", "out[2] = G2 / S;"),
    ("B_small = B in the estimate", "(double)B, 1.0, out + 2)", "(double)B, 2.0, out + 2)"),
]


def _pin_calls():
    """Every pin test as a zero-argument callable (parametrized ones expanded by hand)."""
    calls = [pins.test_hand_worked_example_exact,
             pins.test_finite_differences_dx_dgamma_dbeta_and_per_example,
             pins.test_stats_match_library, pins.test_batch_of_one_norm_equals_big_norm,
             pins.test_d2_eps0_dx_vanishes, pins.test_constant_row_is_finite,
             pins.test_identical_examples_have_zero_noise,
             pins.test_estimators_equal_sample_covariance_trace,
             pins.test_half_identical_examples_closed_form,
             pins.test_T1_reduces_to_elementwise_product_form, pins.test_equivariances,
             pins.test_eq4_eq5_exact_on_noise_model_moments, pins.test_workload_magnitudes]
    for shape in [(3, 7, 33), (5, 1, 16)]:
        calls.append(lambda shape=shape: pins.test_library_autograd_each_example_alone_and_whole_batch(shape))
    for eps in (0.0, 1e-5):
        calls.append(lambda eps=eps: pins.test_dx_row_invariants(eps))
    return calls


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_fails_some_pin(name, old, new, tmp_path):
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation target not found: {old!r}"
    mutated = tmp_path / "mutated.c"
    mutated.write_text(text.replace(old, new, 1))
    lib_path = tmp_path / "libmutated.so"
    subprocess.run(["gcc", "-O1", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off", "-o",
                    str(lib_path), str(mutated), "-lm"], check=True)
    real = oracle._load()
    caught = []
    try:
        oracle._lib = oracle._bind(ctypes.CDLL(str(lib_path)))
        for call in _pin_calls():
            try:
                call()
            except (AssertionError, ValueError, ZeroDivisionError, FloatingPointError):
                caught.append(getattr(call, "__name__", "parametrized"))
    finally:
        oracle._lib = real
    assert caught, f"no pin noticed the planted mistake: {name}"


def test_the_unmutated_oracle_passes_the_same_calls():
    for call in _pin_calls():
        call()
