"""Do the pins of the scheduler-side oracle bite?  Each case plants one plausible mistake in a
COPY of oracle/sched_oracle.py's source (executed as a throw-away module, CPU only) and runs the
pins of test_sched_oracle_pins.py against the copy: at least one must fail, and the unmodified
copy must pass them all.
"""
import os
import types

import numpy as np
import pytest

import oracle
import test_sched_oracle_pins as pins

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "sched_oracle.py")

MUTANTS = {
    "normaliser_is_first_change_not_largest": ("run = np.maximum.accumulate(np.abs(d))", "run = np.full(len(d), abs(d[0]) if len(d) else 0.0)"),
    "normaliser_signed_maximum": ("run = np.maximum.accumulate(np.abs(d))", "run = np.maximum.accumulate(d)"),
    "change_sign_flipped": ("d = L[:-1] - L[1:]", "d = L[1:] - L[:-1]"),
    "weights_favour_old_points": ("w = gamma ** np.arange(m - 1, -1, -1, dtype=np.float64)", "w = gamma ** np.arange(m, dtype=np.float64)"),
    "window_takes_oldest_points": ("L = L[-window:]", "L = L[:window]"),
    "sublinear_without_quadratic_term": ("A = np.stack([t * t, t, np.ones_like(t)], axis=1)", "A = np.stack([0 * t, t, np.ones_like(t)], axis=1)"),
    "sublinear_transform_not_inverted": ("f = 1.0 / lin + off", "f = lin + off"),
    "geometric_uses_log10_exp": ("u = np.log(g)", "u = np.log10(g)"),
    "offset_above_the_minimum": ("off = lo - span * 10.0 ** e\n        p, sse = _fit_for_offset(cls, t, L, w, off)\n        if sse < best[0]:\n            best = (sse, e, off, p)\n    if best[1] is None:",
                                 "off = lo + span * 10.0 ** e\n        p, sse = _fit_for_offset(cls, t, L, w, off)\n        if sse < best[0]:\n            best = (sse, e, off, p)\n    if best[1] is None:"),
    "no_refinement_level": ("for g in range(N_CAND):                # level 2", "for g in range(0):                # level 2"),
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
    for prm in [(0.002, 0.05, 1.2, 0.3), (0.0, 0.08, 0.5, 2.0), (0.01, 0.0, 2.0, 0.05)]:
        yield pins.test_exact_sublinear_curve_is_extrapolated, prm
    yield pins.test_exact_geometric_curve_is_extrapolated, ()
    yield pins.test_prediction_commutes_with_affine_maps_of_the_loss, ()
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
