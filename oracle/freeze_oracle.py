"""CPU oracle of the layer-freezing decision (test infrastructure only: tests,
smoke() and bench.py's cpu_baseline may import it; the product never does).

Section 4.2 of the paper ("How to Decide Layer Freezing") in words: the scores of
the frontmost active module are smoothed with a moving average over the last W
evaluations (Eq. 2), a straight line is fitted to the last W smoothed values, and
when its slope has stayed below a tolerance T for W evaluations in a row the
module is frozen and the next one is watched; when the learning rate has dropped
by a factor of ten since the first freeze, everything is unfrozen and W is
halved.

This file evaluates that description as a batch computation over a whole series
of scores: the series is cut into "watches" (the stretch during which one module
is the frontmost one); inside a watch every quantity is an array over its
evaluations - trailing means from cumulative sums, slopes as weighted means of the
successive differences of each trailing window, run lengths of consecutive
stationary evaluations - and the
watch ends at the first evaluation where a run reaches W (freeze) or the
learning-rate condition holds (unfreeze).  There is no per-evaluation state
machine here; the library's controller, which is one, is compared with this.

Readings taken where the text is silent or at odds with itself:
  * Eq. 2: mean of the last min(W, count) scores of the watch (as printed it sums
    W + 1 terms over W and divides by zero at the first one).
  * The fitted window: the last min(max(W, 2), count) smoothed values against
    0, 1, 2, ... (a line needs two points, also when W = 1); the first evaluation of
    a watch has no slope.
  * Stationary means |slope| < T (as printed, slope < T, a steeply falling curve
    would count).
  * Without a given tolerance, T = 20 % of the largest |slope| among the watch's first
    three slopes, and no evaluation before T is known counts as stationary.
  * The evaluation after W stationary ones in a row freezes the module (its score is
    not used); the last module is never frozen.
  * "Dropped over a factor of 10": lr <= 0.1 * lr_ref * (1 + 1e-12), lr_ref = the
    rate at the evaluation that froze the first module; then all modules are
    unfrozen, the first is watched again and W becomes max(1, W // 2).
"""
from __future__ import annotations

from collections import namedtuple

import numpy as np

NONE, FREEZE, UNFREEZE_ALL = 0, 1, 2

# what one evaluation decided: action, frontmost active module afterwards, run of stationary evaluations,
# window in force afterwards, smoothed score / slope / tolerance (None where there is none)
Evaluation = namedtuple("Evaluation", "action front stale W smoothed slope T")


def trailing_means(x, W):
    """mean of the last min(W, i + 1) values, for every i"""
    c = np.concatenate(([0.0], np.cumsum(np.asarray(x, np.float64))))
    i = np.arange(1, len(x) + 1)
    lo = np.maximum(i - W, 0)
    return (c[i] - c[lo]) / (i - lo)


def trailing_slopes(y, W):
    """least-squares slope of the last m = min(max(W, 2), i + 1) values against 0, 1, 2, ...; NaN at i = 0.
    For equally spaced abscissae the least-squares slope is a weighted mean of the successive differences,
    slope = sum_k w_k (y[k + 1] - y[k]),  w_k = 6 (k + 1) (m - 1 - k) / (m (m^2 - 1)),  k = 0 .. m - 2
    (the weights sum to one; a constant window has slope exactly 0)."""
    y = np.asarray(y, np.float64)
    steps = np.diff(y)
    out = np.full(len(y), np.nan)
    span = max(W, 2)
    for i in range(1, len(y)):
        m = min(span, i + 1)
        k = np.arange(m - 1, dtype=np.float64)
        w = 6.0 * (k + 1.0) * (m - 1.0 - k) / (m * (m * m - 1.0))
        out[i] = float(np.dot(w, steps[i - (m - 1):i]))
    return out


def run_lengths(flags):
    """for every i the number of consecutive True values ending at i"""
    out = np.zeros(len(flags), np.int64)
    run = 0
    for i, f in enumerate(flags):
        run = run + 1 if f else 0
        out[i] = run
    return out


def decide(scores, lrs, n_modules, W, T=0.0, lr_annealing=True):
    """The decisions for a series of scores of the frontmost module (scores[i] at learning rate lrs[i])."""
    scores = np.asarray(scores, np.float64)
    lrs = np.asarray(lrs, np.float64)
    n = len(scores)
    out = [None] * n
    start, front, lr_ref = 0, 0, None
    while start < n:
        m = n - start
        watched = front < n_modules - 1                    # the last module is never frozen
        smoothed = trailing_means(scores[start:], W) if watched else np.full(m, np.nan)
        slopes = trailing_slopes(smoothed, W) if watched else np.full(m, np.nan)
        tol = np.full(m, np.nan)
        if T > 0:
            tol[:] = T                                         # a given tolerance is known throughout
        elif watched and m > 3:
            tol[3:] = 0.2 * np.max(np.abs(slopes[1:4]))        # known from the third slope on
        with np.errstate(invalid="ignore"):
            stationary = np.abs(slopes) < tol                  # False wherever a slope or T is missing
        runs = run_lengths(stationary)
        hits = np.nonzero(runs >= W)[0]
        freeze_at = int(hits[0]) + 1 if watched and len(hits) and hits[0] + 1 < m else None
        # the learning-rate condition can hold from the watch's start (front > 0, reference known)
        drop_at = None
        if lr_annealing and front > 0 and lr_ref is not None:
            d = np.nonzero(lrs[start:] <= 0.1 * lr_ref * (1 + 1e-12))[0]
            drop_at = int(d[0]) if len(d) else None
        end = min(v for v in (freeze_at, drop_at, m) if v is not None)
        for i in range(end):
            out[start + i] = Evaluation(NONE, front, int(runs[i]), W,
                                        None if np.isnan(smoothed[i]) else float(smoothed[i]),
                                        None if np.isnan(slopes[i]) else float(slopes[i]),
                                        None if np.isnan(tol[i]) else float(tol[i]))
        if end == m:
            break
        i = end
        if freeze_at is not None and end == freeze_at:
            if front == 0:
                lr_ref = float(lrs[start + i])
            front += 1
            ev = Evaluation(FREEZE, front, 0, W, None, None, T if T > 0 else None)
            if lr_annealing and lrs[start + i] <= 0.1 * lr_ref * (1 + 1e-12):     # the same evaluation may unfreeze
                front, W, lr_ref = 0, max(1, W // 2), None
                ev = Evaluation(UNFREEZE_ALL, 0, 0, W, None, None, T if T > 0 else None)
        else:
            front, W, lr_ref = 0, max(1, W // 2), None
            ev = Evaluation(UNFREEZE_ALL, 0, 0, W,
                            None if np.isnan(smoothed[i]) else float(smoothed[i]),
                            None if np.isnan(slopes[i]) else float(slopes[i]), T if T > 0 else None)
        out[start + i] = ev
        start += i + 1
    return out
