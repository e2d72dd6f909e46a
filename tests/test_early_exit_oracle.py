"""Pins for the early-exit oracle (paper Sec. 4.1 Algorithm "Loss-Aware Pattern Detection", Sec. 4.2): closed forms of
the EMA and of the regression slope, hand-worked decision sequences with the paper's detector parameters
(w = 2, p = 2, tau_gap = 0.1, tau_slope = 0.001; Sec. 8.3) and the ceil of the warmup selection."""
import math

import numpy as np
import pytest

from oracle import early_exit_oracle as ee

P = ee.Params(alpha=0.5, w=2, tau_slope=1e-3, tau_gap=0.1, p_div=2, p_ovf=2)


def test_ema_closed_form():
    # lhat_t = alpha sum_{j<t} (1-alpha)^j l_{t-j} + (1-alpha)^t l_0
    rng = np.random.default_rng(0)
    l = rng.uniform(0.5, 3.0, size=9)
    for alpha in (0.1, 0.5, 0.9):
        got = ee.ema_series(l, alpha)
        for t in range(len(l)):
            want = (1 - alpha) ** t * l[0] + sum(alpha * (1 - alpha) ** j * l[t - j] for j in range(t))
            assert got[t] == pytest.approx(want, rel=1e-13)
    assert ee.ema_series([2.0] * 5, 0.3) == [2.0] * 5                   # a constant stays put


def test_slope_closed_forms():
    assert ee.linreg_slope([1.0, 1.25]) == pytest.approx(0.25, abs=1e-14)            # w = 2: the difference
    x = np.arange(7.0)
    assert ee.linreg_slope(3.0 - 0.4 * x) == pytest.approx(-0.4, abs=1e-13)         # exact line
    y = np.array([0.3, 1.1, 0.2, 2.5, 1.9])
    xb, yb = x[:5].mean(), y.mean()
    assert ee.linreg_slope(y) == pytest.approx(((x[:5] - xb) * (y - yb)).sum() / ((x[:5] - xb) ** 2).sum(), rel=1e-12)
    assert ee.linreg_slope(y[::-1]) == pytest.approx(-ee.linreg_slope(y), rel=1e-12)  # reversal flips the sign
    assert ee.linreg_slope(y + 7.0) == pytest.approx(ee.linreg_slope(y), rel=1e-12)   # offsets do not matter
    rng = np.random.default_rng(3)
    for w in (2, 3, 5, 16):                                                              # the library's least-squares fit
        z = rng.uniform(0.1, 4.0, size=w)
        assert ee.linreg_slope(z) == pytest.approx(np.polyfit(np.arange(w, dtype=np.float64), z, 1)[0], rel=1e-10, abs=1e-12)
    assert ee.linreg_slope([2.0, 2.25]) == 0.25 and ee.linreg_slope([5.0]) == 0.0      # exact for w = 2


def _run(train_per_eval, val, params=P):
    """One training loss per evaluation step; returns the status after every evaluation."""
    m = ee.Monitor(1, params)
    out = []
    for t, v in zip(train_per_eval, val):
        m.train_loss(0, t)
        out.append(m.val_loss(0, v))
    return out, m.a[0]


def test_divergence_needs_p_consecutive_evaluations_of_both_slopes():
    # alpha = 1 makes lhat the raw loss.  Both curves rise by 0.01 per evaluation; val stays within the gap threshold.
    p = ee.Params(alpha=1.0, w=2, tau_slope=1e-3, tau_gap=0.1, p_div=2, p_ovf=2)
    st, a = _run([1.00, 1.01, 1.02, 1.03], [1.00, 1.01, 1.02, 1.03], p)
    # eval 0: history too short; eval 1: first window, cnt 1; eval 2: cnt 2 -> exit
    assert st == [ee.CONTINUE, ee.CONTINUE, ee.DIVERGING, ee.DIVERGING]
    # a dip of the training slope at the third evaluation resets the counter; two more rising windows are needed
    st, _ = _run([1.00, 1.01, 1.00, 1.01, 1.02], [1.00, 1.01, 1.02, 1.03, 1.04], p)
    assert st == [0, 0, 0, 0, ee.DIVERGING]
    # a rising validation loss alone is not divergence (training keeps falling); the gap is too small to be overfitting
    st, _ = _run([1.00, 0.99, 0.98, 0.97], [1.00, 1.01, 1.02, 1.03], p)
    assert st == [0, 0, 0, 0]
    # slopes exactly at the threshold count (>=)
    q = ee.Params(alpha=1.0, w=2, tau_slope=0.25, tau_gap=10.0, p_div=1, p_ovf=2)
    st, _ = _run([1.0, 1.25], [2.0, 2.25], q)
    assert st == [0, ee.DIVERGING]


def test_overfitting_gap_ratio_is_strict_and_patient():
    p = ee.Params(alpha=1.0, w=2, tau_slope=1e-3, tau_gap=0.1, p_div=2, p_ovf=2)
    # train falls, val 20 % above it for two evaluations in a row -> exit at the second, best val was evaluation 0
    st, a = _run([1.0, 0.9, 0.8], [1.0, 1.08, 0.97], p)          # gaps: 0, 0.2, 0.2125
    assert st == [0, 0, ee.OVERFITTING] and a.best_eval == 2 and a.best_val == 0.97
    # a gap of exactly tau does not count (g > tau)
    st, _ = _run([1.0, 1.0, 1.0], [1.1, 1.1, 1.1], ee.Params(alpha=1.0, w=3, tau_gap=0.1 + 1e-12, p_ovf=1))
    assert st == [0, 0, 0]
    # one evaluation back under the threshold resets the patience
    st, _ = _run([1.0, 0.9, 0.9, 0.9, 0.9], [1.0, 1.08, 0.95, 1.08, 1.08], p)
    assert st == [0, 0, 0, 0, ee.OVERFITTING]


def test_divergence_is_tested_before_overfitting():
    p = ee.Params(alpha=1.0, w=2, tau_slope=1e-3, tau_gap=0.1, p_div=1, p_ovf=1)
    st, _ = _run([1.0, 1.1], [1.0, 1.5], p)     # both rise, and the gap is 36 %
    assert st == [0, ee.DIVERGING]


def test_ema_feeds_the_gap_not_the_raw_loss():
    # alpha = 0.5: lhat after losses 2, 1 is 1.5; val 1.6 is 6.7 % above lhat (no exit) although 60 % above the raw loss
    m = ee.Monitor(1, ee.Params(alpha=0.5, w=5, tau_gap=0.1, p_ovf=1))
    m.train_loss(0, 2.0); m.train_loss(0, 1.0)
    assert m.a[0].lhat == 1.5 and m.val_loss(0, 1.6) == ee.CONTINUE
    assert m.val_loss(0, 1.66) == ee.OVERFITTING              # (1.66 - 1.5) / 1.5 = 0.1067


@pytest.mark.parametrize("ratio,n,k", [(0.25, 8, 2), (0.25, 10, 3), (0.25, 1, 1), (0.1, 30, 3), (0.3, 10, 3),
                                        (1.0, 5, 5), (0.0, 5, 0), (0.25, 0, 0), (0.07, 100, 7), (0.29, 100, 29)])
def test_keep_count_is_the_ceiling_of_the_exact_product(ratio, n, k):
    assert ee.keep_count(ratio, n) == k


def test_warmup_selection_ranks_survivors_only():
    m = ee.Monitor(6, ee.Params(alpha=1.0, w=2, tau_slope=1e-3, tau_gap=0.1, p_div=1, p_ovf=1))
    vals = [0.9, 0.5, 0.7, 0.5, 2.0, 0.6]
    for i, v in enumerate(vals):
        m.train_loss(i, 1.0)
        m.val_loss(i, v)
    assert m.a[4].status == ee.OVERFITTING               # exited during warmup: not ranked
    st = m.warmup_select(0.25)                           # 5 survivors -> keep ceil(1.25) = 2: adapters 1 and 3 (tie, in order)
    assert st == [ee.UNDERPERFORMING, ee.CONTINUE, ee.UNDERPERFORMING, ee.CONTINUE, ee.OVERFITTING, ee.UNDERPERFORMING]


def _paper_settings():
    import os
    vals, keeps = {}, []
    with open(os.path.join(os.path.dirname(__file__), "golden", "early_exit_paper_settings.txt")) as f:
        for line in f:
            parts = line.split()
            if not parts or parts[0].startswith("#"):
                continue
            if parts[0] == "keep":
                keeps.append((int(parts[1]), int(parts[2])))
            else:
                vals[parts[0]] = float(parts[1])
    return vals, keeps


def test_paper_detector_settings_and_sweep_sizes():
    v, keeps = _paper_settings()
    for n, k in keeps:                                    # 25 % of the paper's sweep sizes
        assert ee.keep_count(v["select_ratio"], n) == k
    # with the paper's settings a job whose two curves rise by more than tau_slope per evaluation leaves at the
    # third evaluation (two windows of two values), one whose validation loss sits 11 % above training at the second
    p = ee.Params(alpha=1.0, w=int(v["window"]), tau_slope=v["tau_slope"], tau_gap=v["tau_gap"],
                  p_div=int(v["patience_div"]), p_ovf=int(v["patience_ovf"]))
    st, _ = _run([1.000, 1.002, 1.004], [1.000, 1.002, 1.004], p)
    assert st == [ee.CONTINUE, ee.CONTINUE, ee.DIVERGING]
    st, _ = _run([1.0, 1.0], [1.11, 1.11], p)
    assert st == [ee.CONTINUE, ee.OVERFITTING]
    st, _ = _run([1.0, 1.0, 1.0], [1.09, 1.09, 1.09], p)
    assert st == [0, 0, 0]


def test_non_finite_losses_are_divergence_decided_at_once():
    # hand-worked: a NaN / Inf loss never enters the average or the histories, the adapter is out from that report on,
    # and the others (and the warmup ranking) are not disturbed by it
    m = ee.Monitor(4, ee.Params(alpha=0.5, w=2, tau_slope=1e-3, tau_gap=10.0, p_div=2, p_ovf=2))
    for i in range(4):
        m.train_loss(i, 1.0)
    m.train_loss(0, float("nan"))
    assert m.a[0].status == ee.DIVERGING and m.a[0].lhat == 1.0
    assert m.val_loss(0, 0.5) == ee.DIVERGING and m.a[0].hist_val == []
    assert m.val_loss(1, float("inf")) == ee.DIVERGING and m.a[1].hist_val == [] and m.a[1].best_eval == -1
    m.train_loss(1, 0.3)                                  # ignored: the decision is final
    assert m.a[1].lhat == 1.0
    assert m.val_loss(2, 0.9) == ee.CONTINUE and m.val_loss(3, 0.8) == ee.CONTINUE
    assert m.warmup_select(0.5) == [ee.DIVERGING, ee.DIVERGING, ee.UNDERPERFORMING, ee.CONTINUE]
