"""CPU oracle of the layer-freezing decision (test infrastructure only: tests,
smoke() and bench.py's cpu_baseline may import it; the product never does).

Follows Section 4.2 "How to Decide Layer Freezing" of the paper: the moving
average of Eq. 2, the windowed least-squares slope, the stale counter and the
freeze / unfreeze steps of Algorithm 1, in the paper's order and notation
(pList, staleCounter, W, T, l).  Plain Python and numpy float64; the slope is
the textbook least-squares estimate sum((x - mean x)(y - mean y)) /
sum((x - mean x)^2), which is exactly 0 for a constant history.

Readings taken where the text is silent or at odds with itself:
  * Eq. 2 is read as the mean of the last min(W, count) plasticity values (as
    printed it sums W + 1 terms over W and divides by i = 0 at the first one).
  * windowLinearFit fits the last min(max(W, 2), len(pList)) smoothed values
    against 0, 1, 2, ... (a line needs two points, also when W = 1); with a
    single value there is no slope and the counter is reset.
  * The stale test is |s| < T (as printed, s < T, a steeply falling curve
    would count as stationary).
  * T = 20 % of the largest |slope| among a module's first three slope readings
    when no tolerance is given; nothing is counted before it is known.
  * The learning rate has "dropped over a factor of 10" when
    lr <= 0.1 * lr_ref * (1 + 1e-12), lr_ref being the rate at which the
    frontmost module was frozen; then every module is unfrozen, l returns to the
    first module and W is halved (integer division, at least 1).
  * A frozen module is replaced by the next one with empty history; the last
    module is never frozen.
"""
from __future__ import annotations

import numpy as np

NONE, FREEZE, UNFREEZE_ALL = 0, 1, 2


class FreezeOracle:
    def __init__(self, n_modules: int, W: int, T: float = 0.0, lr_annealing: bool = True):
        self.n_modules, self.W, self.T_user, self.lr_annealing = n_modules, W, T, lr_annealing
        self.l = 0
        self.lr_ref = None
        self._new_module()

    def _new_module(self):
        self.raw = []                 # P_i of the monitored module
        self.pList = []               # smoothed values
        self.staleCounter = 0
        self.first_slopes = []
        self.T = self.T_user if self.T_user > 0 else None

    def smoothPlasticity(self, p):
        self.raw.append(float(p))
        window = self.raw[-min(self.W, len(self.raw)):]
        return float(np.sum(np.asarray(window, np.float64)) / len(window))

    def windowLinearFit(self):
        y = np.asarray(self.pList[-min(max(self.W, 2), len(self.pList)):], np.float64)
        if len(y) < 2:
            return None
        x = np.arange(len(y), dtype=np.float64)
        dx, dy = x - x.mean(), y - y.mean()
        return float((dx * dy).sum() / (dx * dx).sum())

    def checkPlasticity(self, p, lr):
        """One evaluation: plasticity p of the frontmost active module at learning
        rate lr.  Returns (action, l, smoothed, slope)."""
        action, smoothed, s = NONE, None, None
        if self.l < self.n_modules - 1:           # "assert l is not the last layer"
            if self.staleCounter < self.W:
                smoothed = self.smoothPlasticity(p)
                self.pList.append(smoothed)
                s = self.windowLinearFit()
                if s is None:
                    self.staleCounter = 0
                else:
                    if self.T is None:
                        self.first_slopes.append(abs(s))
                        if len(self.first_slopes) == 3:
                            self.T = 0.2 * max(self.first_slopes)
                    if self.T is not None and abs(s) < self.T:
                        self.staleCounter += 1
                    else:
                        self.staleCounter = 0
            else:
                if self.l == 0:
                    self.lr_ref = lr
                self.l += 1
                self._new_module()
                action = FREEZE
        if self.lr_annealing and self.l > 0 and self.lr_ref is not None and lr <= 0.1 * self.lr_ref * (1 + 1e-12):
            self.l = 0
            self.W = max(1, self.W // 2)
            self.lr_ref = None
            self._new_module()
            action = UNFREEZE_ALL
        return action, self.l, smoothed, s
