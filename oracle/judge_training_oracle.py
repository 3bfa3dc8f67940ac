"""CPU fp64 oracle for training the judge verifier (paper Sec. 3.4 "Verifier Training" and
appendix "Training Logistic Regressor").

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the benchmark's cpu_baseline leg,
never by the product path; shares no code with the HIP library.

What the paper fixes: the verifier is a logistic regression on the target's hidden state; an L2
regularisation parameter C is searched over 10 logarithmically spaced values from 1e-3 to 1e2; the
model with the best ROC-AUC is kept; the inference threshold theta is the one with the best F1 (the
"-F" variant) or the best recall (the "-R" variant) on held-out data.

Readings of what it leaves open (each listed in the design notes):
  T1  "C" is the usual inverse regularisation strength: minimise
          f(w, b) = 1/2 |w|^2 + C * sum_i log(1 + exp(-t_i (w.h_i + b))),   t_i = 2 y_i - 1,
      with an unpenalised bias and raw (unscaled) features.  f is strictly convex in w, and in b
      when both classes are present, so the optimum is unique: any solver reaches the same (w, b).
  T2  label 1 = acceptable replacement (Sec. 3.3 step 3), score = sigmoid(w.h + b), accepted when
      score > theta (Eq. 5).
  T3  ROC-AUC, F1 and the thresholds are taken on a held-out validation set given by the caller;
      equal AUC keeps the smaller C.
  T4  best F1: over the candidate thresholds {0} and every validation score, predict "acceptable"
      when score > theta (the rule of Eq. 5); F1 of the acceptable class; equal F1 keeps the
      smallest theta.
  T5  best recall: recall alone is maximal at the trivial thresholds, so it is read as "the most
      permissive threshold that still rejects every unacceptable validation token" (recall 1 on the
      tokens that must be rejected, the conservative "-R" variant): theta_R = the largest score
      of an unacceptable validation token.                                          [parity unpinned]

The solver here is a damped Newton iteration on the dense Hessian - the plainest method for this
objective; the library primitive is numpy.linalg.solve.
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import numpy as np

F64 = np.float64


def paper_c_grid() -> np.ndarray:
    """The 10 logarithmically spaced values from 1e-3 to 1e2 (appendix "Training Logistic Regressor")."""
    return np.logspace(-3.0, 2.0, 10)


def objective(H: np.ndarray, y: np.ndarray, C: float, w: np.ndarray, b: float) -> float:
    """f(w, b) of T1."""
    t = 2.0 * np.asarray(y, F64) - 1.0
    z = np.asarray(H, F64) @ w + b
    return float(0.5 * np.dot(w, w) + C * np.sum(np.logaddexp(0.0, -t * z)))


def fit_logistic(H: np.ndarray, y: np.ndarray, C: float, tol: float = 1e-13, max_iter: int = 200) -> Dict[str, object]:
    """The unique minimiser of f (T1) by Newton's method with step halving.
    Stops when the largest gradient entry is below tol * max(1, C * n)."""
    H = np.asarray(H, F64)
    y = np.asarray(y, F64)
    n, d = H.shape
    if not (0 < y.sum() < n):
        raise ValueError("both classes must be present")
    A = np.concatenate([H, np.ones((n, 1))], axis=1)          # [n, d+1]: bias as a constant feature
    reg = np.ones(d + 1); reg[d] = 0.0                        # the bias is not penalised
    x = np.zeros(d + 1)
    t = 2.0 * y - 1.0

    def f_of(x):
        return 0.5 * np.dot(reg * x, x) + C * np.sum(np.logaddexp(0.0, -t * (A @ x)))

    fx = f_of(x)
    for it in range(max_iter):
        z = A @ x
        s = 1.0 / (1.0 + np.exp(-z))                          # P(y = 1)
        g = reg * x + C * (A.T @ (s - y))
        if np.abs(g).max() <= tol * max(1.0, C * n):
            break
        D = s * (1.0 - s)
        Hess = np.diag(reg) + C * (A.T * D) @ A
        step = np.linalg.solve(Hess, -g)
        alpha = 1.0
        slope = float(np.dot(g, step))
        while True:
            x_new = x + alpha * step
            f_new = f_of(x_new)
            # near the optimum the decrease is below the rounding of f: the full Newton step is taken
            if f_new <= fx + 1e-4 * alpha * slope or abs(slope) <= 1e-9 * abs(fx) or alpha < 1e-10:
                break
            alpha *= 0.5
        x, fx = x_new, f_new
    return {"w": x[:d].copy(), "b": float(x[d]), "iterations": it, "objective": float(fx)}


def scores_of(H: np.ndarray, w: np.ndarray, b: float) -> np.ndarray:
    """Verifier(h) = sigmoid(w.h + b) (Eq. 5)."""
    return 1.0 / (1.0 + np.exp(-(np.asarray(H, F64) @ w + b)))


def roc_auc(scores: np.ndarray, y: np.ndarray) -> float:
    """Area under the ROC curve by its definition: the probability that an acceptable token scores above
    an unacceptable one, ties counted half - over all (acceptable, unacceptable) pairs."""
    s = np.asarray(scores, F64)
    y = np.asarray(y).astype(bool)
    pos, neg = s[y], s[~y]
    if pos.size == 0 or neg.size == 0:
        raise ValueError("both classes must be present")
    gt = 0
    eq = 0
    for p in pos:                                               # one row of the pair table at a time
        gt += int(np.count_nonzero(p > neg))
        eq += int(np.count_nonzero(p == neg))
    return (gt + 0.5 * eq) / (pos.size * neg.size)


def confusion_above(scores: np.ndarray, y: np.ndarray, theta: float):
    """(TP, FP, FN) of the rule "acceptable when score > theta"."""
    s = np.asarray(scores, F64)
    y = np.asarray(y).astype(bool)
    pred = s > theta
    return int(np.count_nonzero(pred & y)), int(np.count_nonzero(pred & ~y)), int(np.count_nonzero(~pred & y))


def f1_of(tp: int, fp: int, fn: int) -> float:
    return 0.0 if tp == 0 else 2.0 * tp / (2.0 * tp + fp + fn)


def best_f1_threshold(scores: np.ndarray, y: np.ndarray) -> Dict[str, float]:
    """T4: candidates are 0 and every validation score; the smallest theta among the best."""
    s = np.asarray(scores, F64)
    best_theta, best_f1 = 0.0, f1_of(*confusion_above(s, y, 0.0))
    for theta in np.unique(s):                                  # increasing
        f1 = f1_of(*confusion_above(s, y, float(theta)))
        if f1 > best_f1:
            best_theta, best_f1 = float(theta), f1
    return {"theta": best_theta, "f1": best_f1}


def best_recall_threshold(scores: np.ndarray, y: np.ndarray) -> float:
    """T5: the largest score of an unacceptable validation token (0 if there is none)."""
    s = np.asarray(scores, F64)
    neg = s[~np.asarray(y).astype(bool)]
    return float(neg.max()) if neg.size else 0.0


def train_judge(H_train: np.ndarray, y_train: np.ndarray, H_val: np.ndarray, y_val: np.ndarray,
                C_grid: Sequence[float]) -> Dict[str, object]:
    """Grid search over C, model selection by validation ROC-AUC (T3), thresholds of the kept model."""
    fits: List[Dict[str, object]] = []
    aucs: List[float] = []
    for C in C_grid:
        fit = fit_logistic(H_train, y_train, float(C))
        fits.append(fit)
        aucs.append(roc_auc(scores_of(H_val, fit["w"], fit["b"]), y_val))
    best = int(np.argmax(aucs))                                 # first maximum = smallest C of the grid order given
    s_val = scores_of(H_val, fits[best]["w"], fits[best]["b"])
    f1 = best_f1_threshold(s_val, y_val)
    return {"w": fits[best]["w"], "b": fits[best]["b"], "best_index": best, "auc": np.array(aucs),
            "theta_f1": f1["theta"], "f1": f1["f1"], "theta_recall": best_recall_threshold(s_val, y_val),
            "val_scores": s_val, "fits": fits}
