"""Pins of the judge-training oracle (Sec. 3.4, appendix "Training Logistic Regressor") against things other
than itself: a library logistic regression, first-order optimality by finite differences, closed-form limits,
library ROC-AUC / F1, brute force on thresholds."""
import numpy as np
import pytest
from scipy.optimize import brentq
from sklearn.linear_model import LogisticRegression
from sklearn.metrics import f1_score, roc_auc_score

import synth
from oracle import judge_training_oracle as jt


def _data(seed, n=400, d=24):
    return synth.make_judge_dataset(seed, n, d, shift=1.5)


def test_c_grid_is_the_papers():
    g = jt.paper_c_grid()
    assert len(g) == 10 and g[0] == pytest.approx(1e-3) and g[-1] == pytest.approx(1e2)
    assert np.allclose(g[1:] / g[:-1], 10 ** (5 / 9))           # logarithmic spacing


@pytest.mark.parametrize("C", [1e-3, 0.17, 1.0, 100.0])
def test_fit_matches_library_logistic_regression(C):
    H, y = _data(1)
    fit = jt.fit_logistic(H, y, C)
    lib = LogisticRegression(C=C, tol=1e-12, max_iter=20000, solver="lbfgs").fit(H.astype(np.float64), y)
    assert np.abs(fit["w"] - lib.coef_[0]).max() < 2e-5 * max(1.0, np.abs(lib.coef_).max())
    assert abs(fit["b"] - lib.intercept_[0]) < 2e-5 * max(1.0, abs(lib.intercept_[0]))
    # and it is at least as good a minimiser of the stated objective
    assert fit["objective"] <= jt.objective(H, y, C, lib.coef_[0], float(lib.intercept_[0])) + 1e-9


def test_first_order_optimality_by_finite_differences():
    H, y = _data(2, n=150, d=6)
    C = 0.7
    fit = jt.fit_logistic(H, y, C)
    Hd, t = H.astype(np.float64), 2.0 * y - 1.0

    def f(x):                                                     # the objective retyped from its definition
        z = Hd @ x[:-1] + x[-1]
        return 0.5 * np.sum(x[:-1] ** 2) + C * np.sum(np.log1p(np.exp(-t * z)))

    x0 = np.append(fit["w"], fit["b"])
    eps = 1e-5
    for i in range(x0.size):
        e = np.zeros_like(x0); e[i] = eps
        assert abs((f(x0 + e) - f(x0 - e)) / (2 * eps)) < 1e-6
    rng = np.random.default_rng(0)
    for _ in range(20):                                           # a strict minimum: every nearby point is worse
        assert f(x0 + 1e-3 * rng.standard_normal(x0.size)) > f(x0)


def test_closed_form_cases():
    # strong regularisation: w -> 0 and the bias reproduces the label rate
    H, y = _data(3)
    fit = jt.fit_logistic(H, y, 1e-9)
    assert np.abs(fit["w"]).max() < 1e-6
    assert fit["b"] == pytest.approx(np.log(y.sum() / (len(y) - y.sum())), abs=1e-5)
    # one feature, two mirrored points: b = 0 by symmetry and w solves  w = 2 C a sigmoid(-a w)
    a, C = 1.3, 0.9
    fit = jt.fit_logistic(np.array([[a], [-a]]), np.array([1, 0]), C)
    w_ref = brentq(lambda w: w - 2 * C * a / (1 + np.exp(a * w)), 0.0, 10.0, xtol=1e-14)
    assert fit["b"] == pytest.approx(0.0, abs=1e-10) and fit["w"][0] == pytest.approx(w_ref, abs=1e-10)
    # a dropped or mis-signed label term would move the weight to the other side
    assert fit["w"][0] > 0
    with pytest.raises(ValueError):
        jt.fit_logistic(np.ones((3, 2)), np.array([1, 1, 1]), 1.0)


def test_roc_auc_against_library_and_special_cases():
    rng = np.random.default_rng(4)
    for trial in range(5):
        y = rng.integers(0, 2, 300)
        s = np.round(rng.random(300), 2 if trial % 2 else 8)      # with and without ties
        assert jt.roc_auc(s, y) == pytest.approx(roc_auc_score(y, s), abs=1e-12)
        assert jt.roc_auc(np.exp(3 * s), y) == pytest.approx(jt.roc_auc(s, y), abs=1e-15)   # rank statistic
        assert jt.roc_auc(-s, y) == pytest.approx(1 - jt.roc_auc(s, y), abs=1e-12)
    y = np.array([0, 0, 1, 1])
    assert jt.roc_auc(np.array([0.1, 0.2, 0.8, 0.9]), y) == 1.0
    assert jt.roc_auc(np.array([0.8, 0.9, 0.1, 0.2]), y) == 0.0
    assert jt.roc_auc(np.full(4, 0.5), y) == 0.5


def test_f1_threshold_against_brute_force_and_library():
    rng = np.random.default_rng(5)
    for trial in range(5):
        y = rng.integers(0, 2, 120)
        s = np.round(np.clip(0.5 + 0.25 * (2 * y - 1) * rng.random(120) + 0.2 * rng.standard_normal(120), 0.01, 0.99), 3)
        got = jt.best_f1_threshold(s, y)
        grid = np.arange(0.0, 1.0, 0.0005)                        # finer than the 1e-3 rounding of the scores
        f1s = np.array([f1_score(y, (s > th).astype(int), zero_division=0) for th in grid])
        assert got["f1"] == pytest.approx(f1s.max(), abs=1e-12)
        assert got["f1"] == pytest.approx(f1_score(y, (s > got["theta"]).astype(int)), abs=1e-12)
        # the smallest best threshold: the brute-force first maximiser falls in the same gap between scores
        first = grid[np.argmax(f1s >= f1s.max() - 1e-12)]
        assert ((s > first) == (s > got["theta"])).all()


def test_recall_threshold_properties():
    rng = np.random.default_rng(6)
    y = rng.integers(0, 2, 200)
    s = rng.random(200)
    th = jt.best_recall_threshold(s, y)
    assert not ((s > th) & (y == 0)).any()                        # every unacceptable token is rejected
    lower = s[s < th].max()
    assert ((s > lower) & (y == 0)).any()                         # and no more permissive candidate does that
    assert jt.best_recall_threshold(np.array([0.3, 0.6]), np.array([1, 1])) == 0.0


def test_train_judge_selects_by_validation_auc():
    H, y = _data(7, n=500, d=32)
    Hv, yv = _data(8, n=300, d=32)
    grid = jt.paper_c_grid()
    r = jt.train_judge(H, y, Hv, yv, grid)
    for i, C in enumerate(grid):
        lib = LogisticRegression(C=C, tol=1e-12, max_iter=20000).fit(H.astype(np.float64), y)
        assert r["auc"][i] == pytest.approx(roc_auc_score(yv, lib.decision_function(Hv.astype(np.float64))), abs=2e-4)
    assert r["best_index"] == int(np.argmax(r["auc"]))
    assert 0.6 < r["auc"].max() < 1.0                             # overlapping classes, as in the paper's ROC figure
    assert np.array_equal(r["w"], r["fits"][r["best_index"]]["w"])
