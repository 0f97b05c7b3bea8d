"""Freeze decision (Section 4.2 "How to Decide Layer Freezing", Eq. 2, Algorithm 1):
pins of the CPU oracle against what the paper and arithmetic fix, then the
library's host-side controller against the oracle on synthetic score series.
No GPU is involved: the controller is host code."""
import math
import os

import numpy as np
import pytest

from oracle import freeze_oracle as fo
from oracle.freeze_oracle import FREEZE, NONE, UNFREEZE_ALL

HERE = os.path.dirname(os.path.abspath(__file__))


def decide(series, n_modules, W, T=0.0, lr=0.1, lr_annealing=True):
    lrs = [lr(i) if callable(lr) else lr for i in range(len(series))]
    return fo.decide(series, lrs, n_modules, W, T, lr_annealing)


# ----------------------------------------------------------------------------- oracle pins

def test_oracle_worked_example():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "freeze_worked_example.txt")) if l[0] != "#"]
    out = decide([float(r[0]) for r in rows] + [0.1], 3, 3, T=0.04)
    for ev, (sc, sm, sl, stale) in zip(out, rows):
        assert ev.action == NONE and ev.front == 0
        assert ev.smoothed == pytest.approx(float(sm), abs=1e-15)
        if sl == "nan":
            assert ev.slope is None
        else:
            assert ev.slope == pytest.approx(float(sl), abs=1e-12)
        assert ev.stale == int(stale)
    last = out[-1]                                           # the run has reached W: the module is frozen
    assert last.action == FREEZE and last.front == 1 and last.smoothed is None and last.stale == 0


@pytest.mark.parametrize("W", [1, 2, 5, 10])
def test_oracle_constant_series_freezes_after_exactly_w_stale_evaluations(W):
    out = decide([0.3] * (3 * W + 8), 4, W, T=1e-6)
    first = [i for i, r in enumerate(out) if r.action == FREEZE]
    # evaluation 0 has no slope; evaluations 1..W are stale; evaluation W+1 freezes
    assert first[0] == W + 1
    assert first[1] == 2 * (W + 1) + 1                      # same again for the next module
    assert out[first[0]].front == 1
    assert [r.stale for r in out[:W + 1]] == list(range(W + 1))


def test_oracle_linear_ramp_never_freezes_and_slope_is_the_ramp():
    W, a = 6, -0.01
    out = decide([1.0 + a * i for i in range(60)], 3, W, T=0.005)
    assert all(r.action == NONE and r.front == 0 for r in out)
    # the moving average of a ramp is the ramp shifted: same slope once the window is full
    for r in out[2 * W:]:
        assert r.slope == pytest.approx(a, rel=1e-9)


def test_oracle_steeply_falling_curve_is_not_stationary():
    """The stale test is on |s|: read as printed (s < T) a falling curve would freeze."""
    out = decide([1.0 - 0.05 * i for i in range(15)], 3, 4, T=0.01)
    assert all(r.action == NONE and r.stale == 0 for r in out)


def test_oracle_moving_average_and_slope_against_definitions():
    """Eq. 2 and the fitted line written out for every evaluation: plain means of slices, and the
    least-squares line of the numerical library (numpy.polyfit) as well as the closed form
    sum((x - mx)(y - my)) / sum((x - mx)^2); the oracle itself uses cumulative sums and a weighted mean
    of successive differences."""
    rng = np.random.default_rng(7)
    W = 5
    series = rng.random(40)
    out = decide(series, 2, W, T=1e-12, lr=1.0)
    sm = []
    for i, ev in enumerate(out):
        lo = max(0, i - W + 1)
        assert ev.smoothed == pytest.approx(sum(series[lo:i + 1]) / (i + 1 - lo), rel=1e-14)
        sm.append(ev.smoothed)
        if i >= 1:
            y = np.array(sm[-min(max(W, 2), len(sm)):])
            x = np.arange(len(y), dtype=np.float64)
            want = ((x - x.mean()) * (y - y.mean())).sum() / ((x - x.mean()) ** 2).sum()
            assert ev.slope == pytest.approx(want, rel=1e-9, abs=1e-15)
            assert ev.slope == pytest.approx(np.polyfit(x, y, 1)[0], rel=1e-9, abs=1e-14)
        else:
            assert ev.slope is None


def test_oracle_automatic_tolerance_is_a_fifth_of_the_largest_early_slope():
    series = [1.0, 0.5, 0.3, 0.25] + [0.25] * 30
    out = decide(series, 3, 4)                   # no tolerance given
    slopes = [abs(r.slope) for r in out[1:4]]
    assert all(r.T is None and r.stale == 0 for r in out[:3])      # two slopes so far: nothing is counted
    assert out[3].T == pytest.approx(0.2 * max(slopes), rel=1e-12)
    assert any(r.action == FREEZE for r in out)


def test_oracle_learning_rate_drop_unfreezes_everything_and_halves_w():
    lr = lambda i: 0.1 if i < 20 else 0.01
    out = decide([0.2] * 40, 4, 6, T=1e-3, lr=lr)
    frozen_at = [i for i, r in enumerate(out) if r.action == FREEZE]
    assert frozen_at[0] == 7 and out[7].front == 1
    assert out[19].action in (NONE, FREEZE) and out[19].front >= 1
    assert out[20].action == UNFREEZE_ALL and out[20].front == 0 and out[20].W == 3
    # after the restart the window is 3: evaluation 21 has no slope, 22..24 are stale, 25 freezes
    assert out[25].action == FREEZE and out[25].front == 1
    # a rate that only fell by a factor of 5 does not unfreeze
    out = decide([0.2] * 40, 4, 6, T=1e-3, lr=lambda i: 0.1 if i < 20 else 0.02)
    assert all(r.action != UNFREEZE_ALL for r in out)


def test_oracle_last_module_is_never_frozen():
    out = decide([0.1] * 30, 2, 2, T=1e-3)
    assert [r.action for r in out].count(FREEZE) == 1 and out[-1].front == 1
    out = decide([0.1] * 10, 1, 2, T=1e-3)
    assert all(r.action == NONE and r.front == 0 and r.smoothed is None and r.slope is None for r in out)


# ----------------------------------------------------------------------------- library vs oracle

def series_bank():
    rng = np.random.default_rng(20220106)
    bank = []
    for k in range(24):
        n = 200
        decay = rng.uniform(0.02, 0.3)
        noise = rng.uniform(0.0, 0.05)
        base = rng.uniform(0.01, 0.2)
        s = base + np.exp(-decay * np.arange(n)) + noise * rng.standard_normal(n) * np.exp(-0.05 * np.arange(n))
        bank.append(s)
    bank.append(np.full(100, 0.25))
    bank.append(1.0 - 0.004 * np.arange(200))
    bank.append(np.zeros(50))
    return bank


@pytest.mark.parametrize("W", [1, 3, 10, 32])
@pytest.mark.parametrize("T", [0.0, 1e-3])
def test_library_controller_matches_oracle(W, T):
    """The library's controller (a state machine fed one score at a time) against the oracle (a batch
    evaluation of the whole series): every action, front index, run length and window equal; smoothed
    values, slopes and the tolerance within rounding."""
    from paper_2201_06227_amd import binding as eg
    for k, series in enumerate(series_bank()):
        lr_of = lambda i: 0.1 * (0.1 ** (i // 70)) if k % 2 == 0 else 0.1
        p32 = [float(np.float32(p)) for p in series]            # scores arrive as fp32
        lrs = [lr_of(i) for i in range(len(series))]
        want = fo.decide(p32, lrs, 5, W, T, True)
        c = eg.FreezeController(5, W, T, True)
        for i, (p, lr, w) in enumerate(zip(p32, lrs, want)):
            d = c.observe(p, lr)
            assert (d.action, d.front, d.stale, d.W) == (w.action, w.front, w.stale, w.W), (k, i)
            if w.smoothed is None:
                assert math.isnan(d.smoothed)
            else:
                assert d.smoothed == pytest.approx(w.smoothed, rel=1e-13, abs=1e-300)
            if w.slope is None:
                assert math.isnan(d.slope)
            else:
                assert d.slope == pytest.approx(w.slope, rel=1e-8, abs=1e-14)
            if w.T is None:
                assert math.isnan(d.T)
            else:
                assert d.T == pytest.approx(w.T, rel=1e-8, abs=1e-14)


def test_library_controller_rejects_bad_arguments():
    from paper_2201_06227_amd import binding as eg
    for bad in [(0, 4, 0.0), (3, 0, 0.0), (3, eg.FREEZE_MAX_W + 1, 0.0), (3, 4, float("nan"))]:
        with pytest.raises(eg.EgeriaError):
            eg.FreezeController(*bad)
    eg.FreezeController(3, eg.FREEZE_MAX_W, 0.0)
