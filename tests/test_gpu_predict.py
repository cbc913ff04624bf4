"""GPU tests of glm_predict_batched against the fp64 scheduler oracle, and of the closed loop
train -> predict -> allocate."""
import numpy as np
import pytest
import torch

import oracle
from oracle import sched_oracle as so
from paper_1802_04819_amd import glm, synth

pytestmark = pytest.mark.gpu

# The fit is a minimisation, so parity is stated on what it minimises.  With E the weighted squared
# error of a curve on the window, evaluated by the oracle's arithmetic:
#   (1) the library's curve and the oracle's are equally good: |E_lib - E_orc| <= 1e-2 E_orc + floor;
#   (2) the library evaluates its own curve correctly: its predictions equal the oracle's `predict`
#       on the library's parameters to 1e-9 of the span, and the error it reports equals E_lib;
#   (3) predictions and normalised reductions agree with the oracle's to 1e-6 of the span (times the
#       sensitivity of the extrapolation, see _amplification) whenever the two errors agree to 1e-6,
#       and to three times the fit's own RMS residual, grown with the square of the extrapolation
#       distance, when they do not (neighbouring dents, see below).
# floor = 1e-24 span^2: on curves that are exact to rounding both errors are ~1e-28 span^2 and their
# ratio means nothing.  1e-2 in (1): a history of fp32 values leaves dents in the floor of the error's
# valley, a few thousandths apart in e and within half a per cent of each other in depth, while the
# walls rise by a factor of four over the same distance; the oracle looks at e every 0.005 and
# refines every dent, the library looks every 0.0235 and follows the lowest sample, so the two can end
# in neighbouring dents.  Measured over 840 random windows: 836
# within 5e-6, three within 5e-3, predictions of all of those within 3e-8 of the span; the remaining
# one (2 % noise, gamma = 0.7, 123 points: ten effective points of noise) ends in another valley, 6 %
# higher.
E_TOL, E_FLOOR, PRED_TOL, SELF_TOL = 1e-2, 1e-24, 1e-6, 1e-9


def _say(msg):
    print(msg, flush=True)


class _Hist:
    """Minimal stand-in for a Job: only loss_hist and hist_len are read by the predictor."""
    def __init__(self, values, device="cuda"):
        self.t = torch.tensor(np.asarray(values, dtype=np.float32), device=device)
        self.c = glm.glm_job_t()
        self.c.loss_hist = self.t.data_ptr()
        self.c.hist_len = len(values)


def _predict(hists, curve, gamma, window, horizon):
    J = len(hists)
    pred = torch.zeros(J, horizon, dtype=torch.float64, device="cuda")
    gain = torch.zeros_like(pred)
    fit = torch.zeros(J, 8, dtype=torch.float64, device="cuda")
    glm.glm_predict_batched(hists, curve, gamma, window, horizon, pred, gain, fit)
    torch.cuda.synchronize()
    return pred.cpu().numpy(), gain.cpu().numpy(), fit.cpu().numpy()


def _check_against_oracle(values32, cls, gamma, window, horizon, pred, gain, fit, tag):
    L = np.asarray(values32, dtype=np.float32).astype(np.float64)
    p_o, g_o, f_o = so.predict_job(L, cls, gamma, window, horizon)
    _, norm = so.normalized_changes(L) if len(L) >= 2 else (None, 0.0)
    assert fit[6] == pytest.approx(norm, rel=1e-15, abs=0), tag
    assert bool(fit[0]) == f_o["ok"], tag
    if not f_o["ok"]:
        assert np.all(pred == f_o["last"]) and np.all(gain == 0), tag
        return
    Lw = L[-window:]
    span = Lw.max() - Lw.min()
    floor = E_FLOOR * span * span
    params = fit[2:5] if cls == so.CLASS_SUBLINEAR else fit[2:4]
    E_lib = so.weighted_error(L, cls, gamma, window, fit[1], params)
    assert abs(E_lib - f_o["sse"]) <= E_TOL * f_o["sse"] + floor, (tag, "depth of the minimum", E_lib, f_o["sse"])
    # (converting the parameters to the units of the losses rounds them; residuals are differences of O(1) values)
    assert abs(fit[5] - E_lib) <= 1e-4 * E_lib + floor, (tag, "reported error", fit[5], E_lib)
    own = dict(f_o); own.update(off=fit[1], p=np.array(params))
    p_own = so.predict(own, horizon)
    assert np.max(np.abs(pred - p_own)) <= SELF_TOL * span, (tag, "own curve", pred, p_own)
    amp = _amplification(f_o, horizon)
    tol = PRED_TOL * span * amp
    if abs(E_lib - f_o["sse"]) > 1e-6 * f_o["sse"] + floor:
        # a neighbouring dent of the valley floor: the two curves differ on the window by about the
        # residual of the fit itself, and h iterations past a window of m points that difference has
        # grown like the square of the distance (the curves are quadratic in t to first order)
        m = len(Lw)
        rms = np.sqrt(f_o["sse"] / np.sum(gamma ** np.arange(m)))
        tol = np.maximum(tol, 3.0 * rms * amp * (1.0 + np.arange(1, horizon + 1) / (m - 1)) ** 2)
    assert np.all(np.abs(pred - p_o) <= tol), (tag, pred, p_o)
    tol2 = np.maximum(tol, np.concatenate([[tol[0]], tol[:-1]]))
    assert np.all(np.abs(gain - g_o) <= tol2 / norm + 1e-12), (tag, gain, g_o)


def _amplification(f, horizon):
    """How much more an extrapolated value moves than the fitted values do when the parameters move
    (>= 1).  A class-I curve with a negative quadratic or linear coefficient has a pole ahead:
    f = 1/q + d, and a change of the coefficients by a fraction eps moves f by eps Q/q^2, with
    Q = |a| t^2 + |b| t + |c|, without bound as q -> 0.  PRED_TOL bounds the movement on the window; the
    tolerance h iterations ahead is scaled by the ratio of that sensitivity to its largest value on the
    window.  Class II: eps (1 + t) exp(p t + q)."""
    m = f["m"]
    tw = np.arange(m, dtype=np.float64) / (m - 1)
    th = (m - 1 + np.arange(1, horizon + 1, dtype=np.float64)) / (m - 1)
    if f["cls"] == so.CLASS_SUBLINEAR:
        a, b, c = f["p"]
        def sens(t):
            q = (a * t + b) * t + c
            Q = abs(a) * t * t + abs(b) * t + abs(c)
            return np.where(q > 0, Q / np.where(q > 0, q, 1.0) ** 2, np.inf)
    else:
        p, q0 = f["p"]
        def sens(t):
            return (1.0 + t) * np.exp(p * t + q0)
    return np.maximum(1.0, sens(th) / np.max(sens(tw)))


def _curves():
    k = np.arange(200, dtype=np.float64)
    rng = np.random.default_rng(0)
    out = []
    out.append(("exact sublinear", 1, 1.0 / (0.002 * k * k + 0.05 * k + 1.2) + 0.3))
    out.append(("noisy sublinear", 1, 1.0 / (0.01 * k + 0.5) + 2.0 + 1e-3 * rng.standard_normal(200)))
    out.append(("exact geometric", 2, 3.0 * 0.9 ** k + 0.25))
    out.append(("noisy geometric", 2, 5.0 * 0.95 ** k + 1.0 + 1e-3 * rng.standard_normal(200)))
    out.append(("geometric fitted as sublinear", 1, 3.0 * 0.9 ** k + 0.25))
    out.append(("increasing", 1, 1.0 + 0.01 * k))
    out.append(("large offset", 1, 1e4 + 1.0 / (0.1 * k + 1.0)))
    out.append(("tiny scale", 2, 1e-6 * 0.8 ** k + 1e-7))
    out.append(("largest change is an increase", 1, 1.0 / (0.01 * k + 0.5) + 2.0 + 4.0 * (k >= 3)))
    out.append(("straight line", 1, 3.0 - 0.01 * k))
    out.append(("straight line as geometric", 2, 3.0 - 0.01 * k))
    out.append(("quadratic and linear terms", 1, 1.0 / (0.01 * k * k + 0.0 * k + 2.0) + 0.05))
    return out


# 20 and 23: lengths at which a coarse search of the offset once settled in the wrong valley
@pytest.mark.parametrize("n", [4, 5, 8, 17, 20, 23, 64, 128, 200])
def test_predictions_match_oracle_on_synthetic_curves(n):
    _say(f"[case] predictor parity, history length {n}")
    curves = _curves()
    hists = [_Hist(c[2][:n]) for c in curves]
    cls = [c[1] for c in curves]
    for gamma, window, horizon in ((0.9, 128, 16), (1.0, 32, 5), (0.7, 128, 64)):
        pred, gain, fit = _predict(hists, cls, gamma, window, horizon)
        for j, (name, c, vals) in enumerate(curves):
            _check_against_oracle(vals[:n].astype(np.float32), c, gamma, window, horizon,
                                  pred[j], gain[j], fit[j], f"{name} n={n} gamma={gamma}")


def test_random_windows_match_oracle():
    """240 seeded random windows: curves of both classes with random parameters, lengths 5..128, noise of
    1e-7 .. 1e-2 of the span, a fifth of them straight lines (nothing of the class), fp32 values."""
    _say("[case] predictor parity on 240 random windows")
    rng = np.random.default_rng(11)
    k = np.arange(200, dtype=np.float64)
    cases = []
    for trial in range(240):
        cls = 1 if trial % 2 == 0 else 2
        n = int(rng.integers(5, 129))
        noise = 10.0 ** rng.uniform(-7, -2) if trial % 7 else 0.0
        if cls == 1:
            L = 1.0 / (10 ** rng.uniform(-4, -1) * k * k + 10 ** rng.uniform(-3, 0) * k + 10 ** rng.uniform(-1, 1)) + rng.uniform(0, 3)
        else:
            L = 10 ** rng.uniform(-1, 1) * rng.uniform(0.5, 0.99) ** k + rng.uniform(0, 3)
        if trial % 5 == 4:
            L = 3.0 - 0.01 * k
        L = L[:n]
        L = (L + noise * (L.max() - L.min()) * rng.standard_normal(n)).astype(np.float32)
        cases.append((cls, L, float(rng.choice([0.7, 0.9, 1.0]))))
    for gamma in (0.7, 0.9, 1.0):
        sub = [c for c in cases if c[2] == gamma]
        pred, gain, fit = _predict([_Hist(c[1]) for c in sub], [c[0] for c in sub], gamma, 128, 16)
        for j, (cls, L, _) in enumerate(sub):
            _check_against_oracle(L, cls, gamma, 128, 16, pred[j], gain[j], fit[j], f"random window {j} gamma={gamma} n={len(L)}")


def test_degenerate_histories():
    _say("[case] predictor: short, flat and single-entry histories")
    vals = [[3.0], [3.0, 2.0], [3.0, 2.0, 1.5], [2.0] * 10, [1.0, 1.0, 1.0, 0.5], [1.0, 1.0, 1.0, 0.5, 0.4]]
    hists = [_Hist(v) for v in vals]
    pred, gain, fit = _predict(hists, 1, 0.9, 128, 4)
    for j, v in enumerate(vals):
        _check_against_oracle(np.float32(v), 1, 0.9, 128, 4, pred[j], gain[j], fit[j], f"degenerate {j}")
    assert np.all(fit[:5, 0] == 0) and np.all(pred[3] == 2.0) and fit[5, 0] == 1


def test_predictor_on_histories_written_by_glm_step_batched():
    _say("[case] predictor on real GPU loss histories: parity and the error at +10 iterations")
    specs = synth.config3_specs(J=24, scale=0.02)
    probs = [synth.config3_job(s, device="cuda") for s in specs]
    jobs = [glm.Job(p.X, p.y, p.w0.clone(), p.loss, p.lam, p.eta, 64) for p in probs]
    ws = glm.alloc_workspace(jobs)
    glm.glm_step_batched(jobs, np.full(24, 30, np.int32), ws)
    torch.cuda.synchronize()
    H = 12
    pred = torch.zeros(24, H, dtype=torch.float64, device="cuda"); gain = torch.zeros_like(pred)
    fit = torch.zeros(24, 8, dtype=torch.float64, device="cuda")
    # gradient descent converges linearly on the strongly convex least-squares jobs (class II) and
    # sublinearly on the others (class I)
    curve = [glm.GLM_CURVE_LINEAR if p.loss == synth.SQUARED else glm.GLM_CURVE_SUBLINEAR for p in probs]
    glm.glm_predict_batched(jobs, curve, 0.9, 128, H, pred, gain, fit)
    torch.cuda.synchronize()
    p_np, g_np, f_np = pred.cpu().numpy(), gain.cpu().numpy(), fit.cpu().numpy()
    for j, job in enumerate(jobs):
        _check_against_oracle(job.history().cpu().numpy(), curve[j], 0.9, 128, H, p_np[j], g_np[j], f_np[j], f"job {j}")
    glm.glm_step_batched(jobs, np.full(24, 10, np.int32), ws)       # what actually happened next
    torch.cuda.synchronize()
    errs = []
    for j, (job, p) in enumerate(zip(jobs, probs)):
        actual = job.loss_hist[39].item()                            # loss 10 iterations after the last fitted one
        errs.append(abs(p_np[j, 9] - actual) / actual)
    errs = np.array(errs)
    smooth = np.array([p.loss != synth.HINGE for p in probs])        # class I assumes a differentiable loss
    print("prediction errors at +10:", np.round(errs, 4), flush=True)
    # Sec. 2 reports under 5 % for the paper's own jobs; on this synthetic mix most jobs are far
    # below that and the worst (least-squares jobs whose error decays at two rates) stay below 10 %
    assert np.mean(errs[smooth] < 0.05) >= 0.7 and np.max(errs[smooth]) < 0.10, errs
    assert np.median(errs) < 0.02


def test_closed_loop_quality_driven_allocation_beats_equal_shares():
    _say("[case] closed loop: train, predict, allocate (greedy) vs equal shares, same total work")
    specs = synth.config3_specs(J=32, scale=0.01)
    specs = [s for s in specs if s.loss != synth.HINGE][:16]
    probs = [synth.config3_job(s, device="cuda") for s in specs]
    J, E, H = len(probs), 6, 16
    C = 4 * J                                                        # iterations per epoch in total

    def run(policy):
        jobs = [glm.Job(p.X, p.y, p.w0.clone(), p.loss, p.lam, p.eta, 64 + E * H) for p in probs]
        # jobs "arrive" with different amounts of progress: job j has already run 4 + 6 j iterations
        ws = glm.alloc_workspace(jobs)
        glm.glm_step_batched(jobs, np.array([4 + (6 * j) % 40 for j in range(J)], np.int32), ws)
        pred = torch.zeros(J, H, dtype=torch.float64, device="cuda"); gain = torch.zeros_like(pred)
        fit = torch.zeros(J, 8, dtype=torch.float64, device="cuda")
        for _ in range(E):
            if policy == "greedy":
                glm.glm_predict_batched(jobs, glm.GLM_CURVE_SUBLINEAR, 0.9, 128, H, pred, gain, fit)
                torch.cuda.synchronize()
                alloc = glm.glm_allocate_greedy(gain.cpu().numpy(), C)
                assert alloc.sum() == C and alloc.min() >= 1
            else:
                alloc = np.full(J, C // J, np.int32)
            glm.glm_step_batched(jobs, alloc, ws)
        torch.cuda.synchronize()
        # normalised loss of a job: where it stands between its first loss and the best loss any run reached
        return [j.history().cpu().numpy() for j in jobs]

    fair, greedy = run("fair"), run("greedy")
    floor = [min(f.min(), g.min()) for f, g in zip(fair, greedy)]
    def mean_norm(hs):
        return float(np.mean([(h[-1] - lo) / (h[0] - lo) for h, lo in zip(hs, floor)]))
    assert mean_norm(greedy) < mean_norm(fair), (mean_norm(greedy), mean_norm(fair))


def test_histories_of_diverged_jobs_give_zero_finite_gains():
    """A job whose loss became NaN or infinite must not poison the epoch: its gains are 0 (so it
    keeps the one unit every job gets) and finite (the allocator rejects anything else)."""
    _say("[case] predictor on histories with NaN, infinities and extreme magnitudes")
    nan, inf = float("nan"), float("inf")
    H = [[nan] * 8, [inf] * 8, [1, nan, 0.5, 0.4, 0.35, 0.33], [1, 0.8, inf, 0.5, 0.4, 0.3], [1, 0.5, 0.25, 0.125, nan],
         [1, 0.9, 0.81, 0.73, -inf], [3e38] * 5, [0.0] * 6,
         [1e30, 5e29, 3e29, 2e29, 1.5e29, 1.2e29], [1e-38, 5e-39, 3e-39, 2e-39, 1e-39], [1, 2, 4, 8, 16, 32]]
    for curve in (glm.GLM_CURVE_SUBLINEAR, glm.GLM_CURVE_LINEAR):
        pred, gain, fit = _predict([_Hist(h) for h in H], curve, 0.9, 128, 8)
        assert np.isfinite(gain).all()
        assert np.all(fit[:8, 0] == 0) and np.all(gain[:8] == 0)          # nothing to fit
        assert np.all(fit[8:10, 0] == 1) and np.all(gain[8:10] > 0) and np.all(gain[8:10] < 1)   # scale does not matter
        alloc = glm.glm_allocate_greedy(gain, 3 * len(H))
        assert alloc.sum() == 3 * len(H) and alloc.min() >= 1 and np.all(alloc[:8] <= alloc[8:10].max())
