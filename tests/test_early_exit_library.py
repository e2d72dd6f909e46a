"""The library's early-exit monitor (host code behind the C ABI) against the oracle: same decisions at the same
evaluation step, same counters and smoothed losses, on synthetic loss curves of the shapes the paper describes
(Sec. 3.2 / Sec. 4.1: converging, diverging, overfitting, noisy) and on values placed at the thresholds."""
import math

import numpy as np
import pytest

from oracle import early_exit_oracle as ee
from paper_2604_05426_amd import binding as ml


def _curves(rng, kind, evals, steps_per_eval):
    """(train losses per step, val loss per evaluation)"""
    n = evals * steps_per_eval
    t = np.arange(n) / n
    noise = rng.normal(0, 0.02, size=n)
    if kind == "converging":
        train = 2.0 * np.exp(-3 * t) + 0.4 + noise
        val = 2.0 * np.exp(-3 * t[steps_per_eval - 1::steps_per_eval]) + 0.45
    elif kind == "diverging":
        knee = rng.uniform(0.2, 0.7)
        train = 1.5 - t + np.where(t > knee, 6 * (t - knee), 0) + noise
        val = (1.5 - t + np.where(t > knee, 6 * (t - knee), 0))[steps_per_eval - 1::steps_per_eval] + 0.05
    elif kind == "overfitting":
        train = 1.8 * np.exp(-4 * t) + 0.1 + noise
        tv = t[steps_per_eval - 1::steps_per_eval]
        val = 1.8 * np.exp(-4 * tv) + 0.15 + np.where(tv > 0.4, 1.5 * (tv - 0.4), 0)
    else:  # noisy plateau around the gap threshold
        train = 1.0 + rng.normal(0, 0.05, size=n)
        val = 1.1 + rng.normal(0, 0.03, size=evals)
    return np.abs(train) + 1e-3, np.abs(val) + 1e-3


@pytest.mark.parametrize("seed", range(12))
def test_monitor_matches_oracle_on_synthetic_curves(seed):
    rng = np.random.default_rng(seed)
    kinds = ["converging", "diverging", "overfitting", "noisy"]
    n = 16
    w = int(rng.integers(2, 6))
    prm = ee.Params(alpha=float(rng.choice([0.05, 0.1, 0.3, 1.0])), w=w, tau_slope=float(rng.choice([1e-3, 1e-2])),
                    tau_gap=float(rng.choice([0.05, 0.1, 0.3])), p_div=int(rng.integers(1, 4)), p_ovf=int(rng.integers(1, 4)))
    evals, spe = 30, int(rng.integers(1, 6))
    curves = [_curves(rng, kinds[i % 4], evals, spe) for i in range(n)]
    orc = ee.Monitor(n, prm)
    mon = ml.Monitor(n, prm.alpha, prm.w, prm.tau_slope, prm.tau_gap, prm.p_div, prm.p_ovf)
    exits = {}
    for e in range(evals):
        for i, (train, val) in enumerate(curves):
            for t in train[e * spe:(e + 1) * spe]:
                orc.train_loss(i, float(t)); mon.train_loss(i, float(t))
            want, got = orc.val_loss(i, float(val[e])), mon.val_loss(i, float(val[e]))
            assert got == want, (seed, i, e)
            st, a = mon.state(i), orc.a[i]
            assert st.ema_train_loss == a.lhat                      # bit for bit: same operations in the same order
            assert (st.count_diverging, st.count_overfitting, st.status) == (a.cnt_div, a.cnt_ovf, a.status)
            assert st.evaluations == len(a.hist_val) and st.best_eval_step == a.best_eval and st.best_val_loss == a.best_val
            if want != ee.CONTINUE:
                exits.setdefault(i, (e, want))
        if e == 4:                                                   # warmup boundary after five evaluations
            assert mon.warmup_select(0.25) == orc.warmup_select(0.25)
    kinds_out = {kinds[i % 4]: reason for i, (_, reason) in exits.items()}
    assert len(exits) > 0 and set(kinds_out.values()) <= {1, 2, 3}
    mon.destroy()


def test_thresholds_decide_alike():
    # values that sit exactly on, just above and just below the two thresholds
    prm = ee.Params(alpha=1.0, w=2, tau_slope=0.25, tau_gap=0.125, p_div=1, p_ovf=1)
    for dv in (0.25, math.nextafter(0.25, 1), math.nextafter(0.25, 0)):
        orc = ee.Monitor(1, prm); mon = ml.Monitor(1, 1.0, 2, 0.25, 0.125, 1, 1)
        for t, v in ((1.0, 1.0), (1.0 + dv, 1.0 + dv)):
            orc.train_loss(0, t); mon.train_loss(0, t)
            assert mon.val_loss(0, v) == orc.val_loss(0, v)
        mon.destroy()
    for gv in (1.125, math.nextafter(1.125, 2), math.nextafter(1.125, 0)):
        orc = ee.Monitor(1, prm); mon = ml.Monitor(1, 1.0, 2, 0.25, 0.125, 1, 1)
        orc.train_loss(0, 1.0); mon.train_loss(0, 1.0)
        assert mon.val_loss(0, gv) == orc.val_loss(0, gv)
        mon.destroy()


def test_monitor_rejects_bad_arguments():
    with pytest.raises(ml.MultiLoraError):
        ml.Monitor(4, 0.0, 2, 1e-3, 0.1, 2, 2)          # alpha
    with pytest.raises(ml.MultiLoraError):
        ml.Monitor(4, 0.1, 1, 1e-3, 0.1, 2, 2)          # window
    m = ml.Monitor(2, 0.1, 2, 1e-3, 0.1, 2, 2)
    with pytest.raises(ml.MultiLoraError):
        m.train_loss(2, 1.0)                            # adapter index
    with pytest.raises(ml.MultiLoraError):
        m.val_loss(0, 1.0)                              # no training loss yet
    with pytest.raises(ml.MultiLoraError):
        m.warmup_select(1.5)
    assert math.isnan(m.state(1).ema_train_loss) and m.state(1).best_eval_step == -1
    m.destroy()


def test_non_finite_losses_decide_alike():
    prm = ee.Params(alpha=0.3, w=3, tau_slope=1e-3, tau_gap=0.2, p_div=2, p_ovf=2)
    rng = np.random.default_rng(99)
    n = 8
    orc = ee.Monitor(n, prm)
    mon = ml.Monitor(n, prm.alpha, prm.w, prm.tau_slope, prm.tau_gap, prm.p_div, prm.p_ovf)
    bad = [float("nan"), float("inf"), -float("inf")]
    for e in range(12):
        for i in range(n):
            for _ in range(3):
                l = float(rng.uniform(0.5, 1.5))
                if rng.random() < 0.04:
                    l = bad[int(rng.integers(0, 3))]
                orc.train_loss(i, l); mon.train_loss(i, l)
            v = float(rng.uniform(0.5, 1.5))
            if rng.random() < 0.04:
                v = bad[int(rng.integers(0, 3))]
            assert mon.val_loss(i, v) == orc.val_loss(i, v), (e, i)
            st, a = mon.state(i), orc.a[i]
            assert st.ema_train_loss == a.lhat and st.status == a.status and st.evaluations == len(a.hist_val)
        if e == 5:
            assert mon.warmup_select(0.5) == orc.warmup_select(0.5)
    assert any(a.status == ee.DIVERGING for a in orc.a)
    mon.destroy()
