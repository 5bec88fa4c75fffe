"""The pins must be able to fail: plant one plausible mistake at a time in a
copy of the oracle's C source (on the CPU), and check that the pin suite
rejects the mutated oracle.  The real oracle is never modified."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

import oracle
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "fb_oracle.c")

MUTATIONS = {
    "beta_uses_v_n_instead_of_v_n_plus_1":
        ("const float *v = emis + (int64_t)(n + 1) * ld;", "const float *v = emis + (int64_t)(n) * ld;"),
    "alpha_multiplies_by_T_not_T_transposed":
        ("semiring_matvec(g->E, g->src, g->dst, g->logw, elo, ehi, klo, khi, x, y, mx);\n            for (int32_t k = klo; k < khi; ++k) a[",
         "semiring_matvec(g->E, g->dst, g->src, g->logw, elo, ehi, klo, khi, x, y, mx);\n            for (int32_t k = klo; k < khi; ++k) a["),
    "beta_multiplies_by_T_transposed":
        ("semiring_matvec(g->E, g->dst, g->src, g->logw, elo, ehi, klo, khi, x, y, mx);\n            for (int32_t k = klo; k < khi; ++k) bn[",
         "semiring_matvec(g->E, g->src, g->dst, g->logw, elo, ehi, klo, khi, x, y, mx);\n            for (int32_t k = klo; k < khi; ++k) bn["),
    "init_dropped":
        ("a[k - klo] = (double)g->init[k] + (double)v[g->pdf[k]];", "a[k - klo] = (double)v[g->pdf[k]];"),
    "first_frame_emission_dropped":
        ("a[k - klo] = (double)g->init[k] + (double)v[g->pdf[k]];", "a[k - klo] = (double)g->init[k];"),
    "final_dropped_from_logz":
        ("logz = lse_pairs(x, g->fin, klo, khi);", "{ double m = ZERO_BAR, s = 0.0; for (int32_t k = klo; k < khi; ++k) if (x[k] > m) m = x[k];\n"
         "      for (int32_t k = klo; k < khi; ++k) s += exp(x[k] - m); logz = m + log(s); }"),
    "beta_starts_at_one_not_final":
        ("bn[k - klo] = (double)g->fin[k];", "bn[k - klo] = 0.0;"),
    "pdf_map_ignored_in_alpha":
        ("a[k - klo] = (double)v[g->pdf[k]] + y[k];", "a[k - klo] = (double)v[k % D] + y[k];"),
    "emission_missing_in_beta":
        ("x[k] = bp[k - klo] + (double)v[g->pdf[k]];", "x[k] = bp[k - klo];"),
    "arc_weight_missing_in_sum":
        ("double t = (double)w[e] + x[tail[e]];\n        y[j] += exp(t - mx[j]);",
         "double t = x[tail[e]];\n        y[j] += exp(t - mx[j]);"),
    "logsumexp_sign":
        ("y[j] += exp(t - mx[j]);", "y[j] += exp(mx[j] - t);"),
    "posterior_not_normalised":
        ("exp(a + b - logz);", "exp(a + b);"),
    "rho_overwrites_instead_of_adding":
        ("rho[(int64_t)n * D + g->pdf[k]] += p;", "rho[(int64_t)n * D + g->pdf[k]] = p;"),
    "lfmmi_sign":
        ("gr[t] -= rho[t];", "gr[t] += rho[t];"),
    "lfmmi_num_uses_den_graph":
        ("logz_num[i] = fb_sequence(&gn, klo, khi, arc_off[b], arc_off[b + 1]", "logz_num[i] = fb_sequence(&gd, 0, Kd < Kb ? Kd : Kb, 0, 0"),
}


def pin_suite():
    pins.test_hand_computed_two_state_example()
    pins.test_brute_force_enumeration(3, 4, 4, 3)
    pins.test_brute_force_enumeration(4, 3, 6, 5)
    pins.test_single_path_chain_closed_form()
    pins.test_constant_emission_markov_chain_closed_form()
    pins.test_invariants("zipf")
    pins.test_lfmmi_matches_separate_runs_and_sums_to_zero()
    pins.test_lfmmi_gradient_finite_difference()


def test_pin_suite_accepts_the_real_oracle():
    pin_suite()


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_pin_suite_rejects_mutated_oracle(name, tmp_path, monkeypatch):
    old, new = MUTATIONS[name]
    text = open(SRC).read()
    assert text.count(old) == 1, "mutation anchor must match exactly once"
    csrc = tmp_path / "mut.c"
    csrc.write_text(text.replace(old, new))
    so = tmp_path / "libmut.so"
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-o", str(so), str(csrc), "-lm"])
    lib = ctypes.CDLL(str(so))
    lib.fbo_forward_backward.restype = ctypes.c_int
    lib.fbo_lfmmi.restype = ctypes.c_int
    lib.fbo_num_threads.restype = ctypes.c_int
    oracle._load()
    monkeypatch.setattr(oracle, "_lib", lib)
    with pytest.raises((AssertionError, FloatingPointError, ValueError)):
        pin_suite()
