"""Do the pins of the scheduler-side oracle bite?  Each case plants one plausible mistake in a
COPY of the oracle's source -- oracle/sched_oracle.py executed as a throw-away module, or
oracle/sched_fit.c compiled into a throw-away library (CPU only) -- and runs the quick pins of
test_sched_oracle_pins.py against the copy: at least one must fail, and the unmodified copies
must pass them all.
"""
import ctypes
import os
import subprocess
import types

import numpy as np
import pytest

import oracle
import test_sched_oracle_pins as pins

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "sched_oracle.py")
SRC_C = os.path.join(ROOT, "oracle", "sched_fit.c")

MUTANTS = {
    "normaliser_is_first_change_not_largest": ("run = np.maximum.accumulate(np.abs(d))", "run = np.full(len(d), abs(d[0]) if len(d) else 0.0)"),
    "normaliser_signed_maximum": ("run = np.maximum.accumulate(np.abs(d))", "run = np.maximum.accumulate(d)"),
    "change_sign_flipped": ("d = L[:-1] - L[1:]", "d = L[1:] - L[:-1]"),
    "window_takes_oldest_points": ("    L = L[-window:]\n    m = len(L)\n    out =", "    L = L[:window]\n    m = len(L)\n    out ="),
    "prediction_starts_at_last_point": ("t = (m - 1 + np.arange(1, H + 1, dtype=np.float64)) / (m - 1)", "t = (m - 1 + np.arange(0, H, dtype=np.float64)) / (m - 1)"),
    "prediction_time_unscaled": ("t = (m - 1 + np.arange(1, H + 1, dtype=np.float64)) / (m - 1)", "t = (m - 1 + np.arange(1, H + 1, dtype=np.float64))"),
    "gain_not_normalised": ("gain = (prev - pred) / norm if norm > 0 else np.zeros(int(horizon))", "gain = (prev - pred) if norm > 0 else np.zeros(int(horizon))"),
    "gain_from_last_loss_not_fit": ("prev = np.concatenate([[fitted_value_at_last(fit)], pred[:-1]])", "prev = np.concatenate([[2 * L[-1] - fitted_value_at_last(fit)], pred[:-1]])"),
    "greedy_starts_from_zero_units": ("a = np.ones(J, dtype=np.int64)\n    left = int(capacity) - J", "a = np.zeros(J, dtype=np.int64)\n    left = int(capacity)"),
    "greedy_looks_at_current_unit": ("if a[j] < H and gain[j, a[j]] > best_g:\n                best_j, best_g = j, gain[j, a[j]]",
                                     "if a[j] < H and gain[j, a[j] - 1] > best_g:\n                best_j, best_g = j, gain[j, a[j] - 1]"),
    "greedy_ties_to_last_job": ("if a[j] < H and gain[j, a[j]] > best_g:", "if a[j] < H and gain[j, a[j]] >= best_g:"),
    "greedy_ignores_cap": ("if a[j] < H and gain[j, a[j]] > best_g:", "if gain[j, min(a[j], H - 1)] > best_g:"),
    "greedy_picks_smallest_gain": ("best_j, best_g = -1, -np.inf\n        for j in range(J):\n            if a[j] < H and gain[j, a[j]] > best_g:",
                                   "best_j, best_g = -1, np.inf\n        for j in range(J):\n            if a[j] < H and gain[j, a[j]] < best_g:"),
}

# mistakes in the C source of the fit
MUTANTS_C = {
    "weights_favour_old_points": ("W.w[i] = pow(gamma, (double)(m - 1 - i));", "W.w[i] = pow(gamma, (double)i);"),
    "error_not_weighted": ("        s += W->w[i] * r * r;", "        s += r * r;"),
    "time_not_scaled": ("W.t[i] = (double)i / (double)(m - 1);", "W.t[i] = (double)i;"),
    "losses_not_normalised": ("W.l[i] = (L[i] - lo) / span;", "W.l[i] = L[i] - lo;"),
    "sublinear_derivative_sign": ("const double dq = -1.0 / (q * q);", "const double dq = 1.0 / (q * q);"),
    "sublinear_without_quadratic_term": ("J[0] = dq * t * t; J[1] = dq * t; J[2] = dq;", "J[0] = 0.0; J[1] = dq * t; J[2] = dq;"),
    "geometric_derivative_misses_time": ("J[0] = E * t; J[1] = E; J[2] = 0.0;", "J[0] = E; J[1] = E; J[2] = 0.0;"),
    "geometric_error_without_offset": ("            f = exp(lin[0] * t + lin[1]) + off;\n        }\n        const double r = f - W->l[i];\n        s +=",
                                       "            f = exp(lin[0] * t + lin[1]);\n        }\n        const double r = f - W->l[i];\n        s +="),
    "offset_above_the_minimum": ("out[1] = lo - span * pow(10.0, best_e);", "out[1] = lo + span * pow(10.0, best_e);"),
    "box_ends_one_span_down": ("kExpLo = -4.0, kExpHi = 2.0;", "kExpLo = -4.0, kExpHi = 0.0;"),
    "no_refinement_of_the_scan": ("while (b - a > kGoldenTol) {", "while (0 * (b - a) > kGoldenTol) {"),
    "worst_valley_wins": ("if (v < best) { best = v;", "if (v > best || !isfinite(best)) { best = v;"),
    "no_gauss_newton": ("for (int it = 0; it < 200; ++it) {", "for (int it = 0; it < 0; ++it) {"),
    "span_not_undone_sublinear": ("out[2] = best_lin[0] / span; out[3] = best_lin[1] / span; out[4] = best_lin[2] / span;",
                                  "out[2] = best_lin[0]; out[3] = best_lin[1]; out[4] = best_lin[2];"),
    "span_not_undone_geometric": ("out[3] = best_lin[1] + log(span);", "out[3] = best_lin[1];"),
}


def _module(old=None, new=None, name="mutant"):
    src = open(SRC).read()
    if old is not None:
        assert src.count(old) == 1, f"mutation site not found exactly once: {old[:40]}"
        src = src.replace(old, new)
    mod = types.ModuleType(name)
    exec(compile(src, name, "exec"), mod.__dict__)
    return mod


def _cases():
    yield pins.test_normalized_changes_hand_example, ()
    yield pins.test_first_normalized_change_is_one_and_values_stay_in_unit_interval, ()
    for prm in pins.SUBLINEAR_CURVES:
        yield pins.test_exact_sublinear_curve_is_extrapolated, prm
    yield pins.test_lengths_at_which_a_neighbouring_valley_is_almost_as_deep, ()
    yield pins.test_exact_geometric_curve_is_extrapolated, ()
    yield pins.test_prediction_commutes_with_affine_maps_of_the_loss, ()
    yield pins.test_the_offset_stays_inside_its_box, ()
    yield pins.test_weights_enter_the_fit, ()
    for cls, n in ((1, 12), (1, 40), (2, 12), (2, 40)):
        yield pins.test_noisy_history_reaches_the_reference_minimum, (cls, n)
    yield pins.test_tenth_next_iteration_of_gradient_descent_within_five_percent, (oracle.LOGISTIC, 0.5, 1)
    yield pins.test_tenth_next_iteration_of_gradient_descent_within_five_percent, (oracle.SQUARED, 0.1, 2)
    yield pins.test_short_or_flat_histories_predict_the_last_loss, ()
    yield pins.test_only_the_window_is_used_and_recent_points_weigh_more, ()
    yield pins.test_greedy_hand_example, ()
    yield pins.test_greedy_is_optimal_for_diminishing_gains_by_brute_force, ()


def _first_failure(mod):
    saved = pins.so
    pins.so = mod
    try:
        for fn, prm in _cases():
            try:
                fn(*prm)
            except (AssertionError, ValueError, IndexError, FloatingPointError, np.linalg.LinAlgError):
                return fn.__name__
            except pytest.fail.Exception:                       # pytest.raises that did not raise
                return fn.__name__
    finally:
        pins.so = saved
    return None


def test_unmodified_copy_passes_every_pin():
    assert _first_failure(_module(name="clean")) is None


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_rejected(name):
    old, new = MUTANTS[name]
    assert _first_failure(_module(old, new, name)) is not None, f"no pin notices: {name}"


def _compile_fit(tmp_path, name, old=None, new=None):
    src = open(SRC_C).read()
    if old is not None:
        assert src.count(old) == 1, f"mutation site not found exactly once: {old[:40]}"
        src = src.replace(old, new)
    c = tmp_path / f"{name}.c"
    lib = tmp_path / f"{name}.so"
    c.write_text(src)
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-o", str(lib), str(c), "-lm"], check=True)
    h = ctypes.CDLL(str(lib))
    dp = ctypes.POINTER(ctypes.c_double)
    h.oracle_fit_curve.restype = ctypes.c_int
    h.oracle_fit_curve.argtypes = [ctypes.c_int, dp, ctypes.c_int, ctypes.c_double, dp]
    return h


def _first_failure_with_fit(lib):
    mod = _module(name="with_fit_copy")
    mod.FIT_LIB = lib
    return _first_failure(mod)


def test_unmodified_copy_of_the_fit_passes_every_pin(tmp_path):
    assert _first_failure_with_fit(_compile_fit(tmp_path, "clean")) is None


@pytest.mark.parametrize("name", sorted(MUTANTS_C))
def test_mutant_of_the_fit_is_rejected(tmp_path, name):
    old, new = MUTANTS_C[name]
    assert _first_failure_with_fit(_compile_fit(tmp_path, name, old, new)) is not None, f"no pin notices: {name}"
