"""CPU oracle for loss-aware early exit -- TEST INFRASTRUCTURE ONLY.

Follows the paper's online pattern detection (Sec. 4.1, Algorithm "Loss-Aware Pattern Detection") and the
warmup-boundary selection (Sec. 4.2), in the paper's notation, one adapter at a time, plain Python floats (fp64):

* training loss is smoothed by an exponential moving average  lhat_t = alpha l_t + (1 - alpha) lhat_{t-1};
* at every evaluation step the current lhat_train and the raw l_val are appended to the two histories, then
  Pattern 1 (divergence): once both histories hold at least w values, the least-squares slopes of the last w values of
      each are taken; cnt_div <- cnt_div + 1 if both slopes >= tau_slope, else 0; exit "diverging" when cnt_div >= p_div;
  Pattern 2 (overfitting): g = (l_val[-1] - lhat_train[-1]) / lhat_train[-1]; cnt_ovf <- cnt_ovf + 1 if g > tau_gap,
      else 0; exit "overfitting" when cnt_ovf >= p_ovf, reporting the evaluation step of the best validation loss;
* Pattern 3 (underperformance), at the warmup boundary only: surviving adapters are ranked by validation loss and the
  best k = ceil(ratio x survivors) are kept.

Readings where the paper is silent (listed in the design notes as well):
  1. lhat_0 = l_0: the first training loss seeds the average.
  2. The histories have one entry per evaluation step, so slopes are per evaluation step (x = 0 .. w-1).
  3. While a history is shorter than w the divergence counter is left unchanged (it is still zero then).
  4. Pattern 1 is tested before Pattern 2, as the algorithm lists them; an adapter that meets both exits as diverging.
  5. g is only defined for lhat_train > 0; otherwise the step counts as "gap not exceeded" (counter reset).
  6. An evaluation with no training loss seen yet is an error (there is no lhat to compare with).
  7. Ranking at the warmup boundary uses each survivor's latest validation loss, ascending; equal losses keep adapter
     order; survivors that have never been evaluated rank last.  k = ceil(ratio x n) is taken on the exact product: a
     product within 1e-9 of an integer counts as that integer (0.1 x 30 must give 3, not 4).
  8. A training or validation loss that is NaN or infinite is the end point of Pattern 1 (the loss has left the number
     line): the adapter exits as diverging at that report; the value enters neither the average nor the histories
     (inside them it would turn every later comparison false, and the warmup ranking would have no order).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

CONTINUE, DIVERGING, OVERFITTING, UNDERPERFORMING = 0, 1, 2, 3


@dataclass
class Params:
    alpha: float = 0.1          # EMA weight of the newest training loss
    w: int = 2                  # regression window (evaluation steps)
    tau_slope: float = 1e-3
    tau_gap: float = 0.1
    p_div: int = 2
    p_ovf: int = 2


def ema_series(losses: Sequence[float], alpha: float) -> List[float]:
    out: List[float] = []
    for l in losses:
        out.append(float(l) if not out else alpha * float(l) + (1.0 - alpha) * out[-1])
    return out


def linreg_slope(y: Sequence[float]) -> float:
    """Slope of the least-squares line through (0, y_0) .. (w-1, y_{w-1}):
    sum_x (x - xbar)(y_x - ybar) / sum_x (x - xbar)^2, sums taken left to right in fp64.  (Thresholds are compared with
    this number, so the formula and its summation order are part of the definition; a window of one value has slope 0.)"""
    w = len(y)
    if w < 2:
        return 0.0
    xbar = (w - 1) / 2.0
    ybar = 0.0
    for v in y:
        ybar += float(v)
    ybar /= w
    num = den = 0.0
    for x, v in enumerate(y):
        num += (x - xbar) * (float(v) - ybar)
        den += (x - xbar) * (x - xbar)
    return num / den


@dataclass
class Adapter:
    lhat: Optional[float] = None
    hist_train: List[float] = field(default_factory=list)
    hist_val: List[float] = field(default_factory=list)
    cnt_div: int = 0
    cnt_ovf: int = 0
    status: int = CONTINUE
    best_val: float = math.inf
    best_eval: int = -1          # 0-based index of the evaluation step with the best validation loss


class Monitor:
    def __init__(self, n: int, params: Params):
        self.p = params
        self.a = [Adapter() for _ in range(n)]

    def train_loss(self, i: int, loss: float) -> None:
        a = self.a[i]
        if a.status != CONTINUE:
            return
        if not math.isfinite(loss):       # reading: a non-finite loss is divergence, decided at once
            a.status = DIVERGING
            return
        a.lhat = float(loss) if a.lhat is None else self.p.alpha * float(loss) + (1.0 - self.p.alpha) * a.lhat

    def val_loss(self, i: int, val: float) -> int:
        a, p = self.a[i], self.p
        if a.status != CONTINUE:
            return a.status
        if a.lhat is None:
            raise ValueError("validation loss before any training loss")
        if not math.isfinite(val):
            a.status = DIVERGING
            return a.status
        a.hist_train.append(a.lhat)
        a.hist_val.append(float(val))
        if val < a.best_val:
            a.best_val, a.best_eval = float(val), len(a.hist_val) - 1
        # Pattern 1
        if len(a.hist_train) >= p.w and len(a.hist_val) >= p.w:
            s_train = linreg_slope(a.hist_train[-p.w:])
            s_val = linreg_slope(a.hist_val[-p.w:])
            a.cnt_div = a.cnt_div + 1 if (s_train >= p.tau_slope and s_val >= p.tau_slope) else 0
            if a.cnt_div >= p.p_div:
                a.status = DIVERGING
                return a.status
        # Pattern 2
        lt = a.hist_train[-1]
        exceeded = lt > 0.0 and (a.hist_val[-1] - lt) / lt > p.tau_gap
        a.cnt_ovf = a.cnt_ovf + 1 if exceeded else 0
        if a.cnt_ovf >= p.p_ovf:
            a.status = OVERFITTING
        return a.status

    def warmup_select(self, ratio: float) -> List[int]:
        """Status of every adapter after the warmup boundary (Pattern 3 applied to the survivors)."""
        alive = [i for i, a in enumerate(self.a) if a.status == CONTINUE]
        ranked = sorted(alive, key=lambda i: (self.a[i].hist_val[-1] if self.a[i].hist_val else math.inf, i))
        k = keep_count(ratio, len(ranked))
        for i in ranked[k:]:
            self.a[i].status = UNDERPERFORMING
        return [a.status for a in self.a]


def keep_count(ratio: float, n: int) -> int:
    x = ratio * n
    r = round(x)
    if abs(x - r) <= 1e-9:
        return int(min(max(r, 0), n))
    return int(min(max(math.ceil(x), 0), n))
