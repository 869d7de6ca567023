"""Are the pins sharp?  Plant one plausible mistake at a time in a COPY of the oracle's C
source (CPU only), build it, and require that at least one pin test fails for it.  The
committed oracle is never modified and the GPU is never involved.
"""
import ctypes
import inspect
import os
import subprocess

import pytest

from oracle import grawa_oracle as orc
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(orc.__file__), "grawa_oracle.c")

# (name, text in the oracle source, planted replacement)
MUTANTS = [
    ("dropped_square", "s += v * v;", "s += v;"),
    ("sumsq_skips_first_element", "for (int64_t i = off[k]; i < off[k + 1]; ++i) {", "for (int64_t i = off[k] + 1; i < off[k + 1]; ++i) {"),
    ("sumsq_ignores_leading_dimension", "double v = widen_at(g, dtype, m * ldg + i);", "double v = widen_at(g, dtype, m * off[L] + i);"),
    ("layer_norm_without_sqrt", "A[m * L + k] = sqrt(S[m * L + k]);", "A[m * L + k] = S[m * L + k];"),
    ("layersum_of_squares", "a += sqrt(S[m * L + k]);", "a += S[m * L + k];"),
    ("flat_without_sqrt", "a = sqrt(a);", ";"),
    ("flat_and_layersum_swapped", "if (mode == ORACLE_NORM_LAYERSUM) {", "if (mode == ORACLE_NORM_FLAT) {"),
    ("normaliser_sums_norms", "z += 1.0 / A[m * G + j];", "z += A[m * G + j];"),
    ("weights_proportional_not_inverse", "1.0 / A[m * G + j]", "A[m * G + j]"),
    ("weights_not_normalised", "beta[m * G + j] = (1.0 / A[m * G + j]) / z;", "beta[m * G + j] = (1.0 / A[m * G + j]);"),
    ("zero_rule_not_shared", "? 1.0 / (double)n0 : 0.0;", "? 1.0 : 0.0;"),
    ("weights_normalised_over_layers", "for (int64_t m = 0; m < K; ++m) z += 1.0 / A[m * G + j];", "for (int64_t m = 0; m < G; ++m) z += 1.0 / A[j * G + m];"),
    ("beta_table_transposed", "s += beta[m * G + layer] * xd[m * n + i];", "s += beta[layer * K + m] * xd[m * n + i];"),
    ("layer_boundary_off_by_one", "off[layer + 1] <= i0 + i", "off[layer + 1] < i0 + i"),
    ("center_ignores_chunk_start", "off[layer + 1] <= i0 + i", "off[layer + 1] <= i"),
    ("pull_swapped", "xd[m * n + i] = (1.0 - lambda) * xd[m * n + i] + lambda * c[i];", "xd[m * n + i] = lambda * xd[m * n + i] + (1.0 - lambda) * c[i];"),
    ("pull_away_from_center", "(1.0 - lambda) * xd[m * n + i] + lambda * c[i];", "(1.0 + lambda) * xd[m * n + i] - lambda * c[i];"),
    ("pull_uses_updated_workers", "xd[m * n + i] = (1.0 - lambda) * xd[m * n + i] + lambda * c[i];", "xd[m * n + i] = (1.0 - lambda) * xd[m * n + i] + lambda * (m ? xd[(m - 1) * n + i] : c[i]);"),
    ("sgd_ascent", "xd[m * n + i] - eta * widen_at", "xd[m * n + i] + eta * widen_at"),
    ("sgd_ignores_chunk_start", "widen_at(g, dtype, m * ldg + i0 + i);", "widen_at(g, dtype, m * ldg + i);"),
    ("load_ignores_chunk_start", "(double)x[m * ldx + i0 + i];", "(double)x[m * ldx + i];"),
    ("load_ignores_leading_dimension", "(double)x[m * ldx + i0 + i];", "(double)x[m * n + i0 + i];"),
    ("bf16_wrong_shift", "<< 16;", "<< 15;"),
    ("prox_swapped", "xd[m * n + i] = (1.0 - w) * xd[m * n + i] + w * c[i];", "xd[m * n + i] = w * xd[m * n + i] + (1.0 - w) * c[i];"),
    ("prox_not_scaled_by_period", "double w = mu / tau;", "double w = mu;"),
    ("momentum_weights_swapped", "g_mvg[i] = gamma * g_mvg[i] + (1.0 - gamma) * g_cur[i];", "g_mvg[i] = (1.0 - gamma) * g_mvg[i] + gamma * g_cur[i];"),
    ("momentum_forgets_history", "g_mvg[i] = gamma * g_mvg[i] + (1.0 - gamma) * g_cur[i];", "g_mvg[i] = (1.0 - gamma) * g_cur[i];"),
    ("bias_correction_missing", "g_est[i] = gamma * g_mvg[i] / denom;", "g_est[i] = gamma * g_mvg[i];"),
    ("bias_correction_wrong_power", "double denom = 1.0 - pow(gamma, (double)t);", "double denom = 1.0 - pow(gamma, (double)(t + 1));"),
    ("estimate_without_leading_gamma", "g_est[i] = gamma * g_mvg[i] / denom;", "g_est[i] = g_mvg[i] / denom;"),
    ("nesterov_without_lookahead", "xd[m * n + i] = xd[m * n + i] - eta * (d + momentum * buf[m * n + i]);", "xd[m * n + i] = xd[m * n + i] - eta * buf[m * n + i];"),
    ("nesterov_decay_dropped", "+ wd * xd[m * n + i];", ";"),
    ("nesterov_buffer_dampened", "buf[m * n + i] = momentum * buf[m * n + i] + d;", "buf[m * n + i] = momentum * buf[m * n + i] + (1.0 - momentum) * d;"),
    ("easgd_center_is_a_noop", "c[i] = (1.0 - rho) * c[i] + rho * (s / (double)K);", "c[i] = (1.0 - rho) * (s / (double)K) + rho * (s / (double)K);"),
    ("easgd_sum_not_mean", "rho * (s / (double)K);", "rho * s;"),
    ("leader_is_largest_loss", "if (loss[m] < loss[best]) best = m;", "if (loss[m] > loss[best]) best = m;"),
    ("leader_last_on_ties", "if (loss[m] < loss[best]) best = m;", "if (loss[m] <= loss[best]) best = m;"),
    ("nonfinite_misses_infinity", "if (!isfinite(A[i])) return 1;", "if (isnan(A[i])) return 1;"),
    ("nonfinite_skips_last_entry", "for (int64_t i = 0; i < n; ++i)\n        if (!isfinite(A[i])) return 1;", "for (int64_t i = 0; i + 1 < n; ++i)\n        if (!isfinite(A[i])) return 1;"),
    ("layer_sum_skips_first", "for (int64_t k = 0; k < L; ++k) a += est[m * L + k];", "for (int64_t k = 1; k < L; ++k) a += est[m * L + k];"),
]

PIN_TESTS = [(n, f) for n, f in inspect.getmembers(pins, inspect.isfunction) if n.startswith("test_")]


def _run_all_pins():
    """Run every pin test in-process; return the names of those that fail."""
    failed = []
    for name, fn in PIN_TESTS:
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        cases = [()]
        if marks:
            argvalues = marks[0].args[1]
            cases = [(v,) for v in argvalues]
        for args in cases:
            try:
                fn(*args)
            except Exception:  # an assertion, or the mutant crashing a check
                failed.append(name)
                break
    return failed


def test_unmutated_oracle_passes_the_harness():
    assert _run_all_pins() == []


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, monkeypatch, name, old, new):
    src = open(SRC).read()
    assert src.count(old) >= 1, "mutant pattern no longer present in the oracle source: %r" % old
    # every occurrence: some mistakes (e.g. inverse vs proportional) touch two lines
    mutated = src.replace(old, new)
    c = tmp_path / "mutant.c"
    so = tmp_path / "mutant.so"
    c.write_text(mutated)
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-w", "-fno-fast-math", "-ffp-contract=off",
                           "-shared", "-fPIC", "-o", str(so), str(c), "-lm"])
    monkeypatch.setattr(orc, "_lib", orc._bind(ctypes.CDLL(str(so))))
    failed = _run_all_pins()
    assert failed, "no pin noticed the planted mistake '%s'" % name
