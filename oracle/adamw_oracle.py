"""CPU oracle for the per-adapter AdamW update -- TEST INFRASTRUCTURE ONLY.

The paper trains every LoRA job with its own optimizer instance (Sec. 5.2: each rank keeps
independent parameters, optimizers and loss trackers per adapter; App. training details: AdamW,
weight decay 0.01, constant learning rate).  The paper's optimizer is a paged 8-bit AdamW; the
quantised state is not part of this build, so the update below is the plain AdamW definition with
decoupled weight decay, in fp64, one adapter matrix at a time:

    m   <- beta1 m + (1 - beta1) g
    v   <- beta2 v + (1 - beta2) g^2
    mh   = m / (1 - beta1^t),   vh = v / (1 - beta2^t)
    th  <- th - lr (mh / (sqrt(vh) + eps) + wd th)

`t` is the 1-based step count of that adapter (adapters that joined later are at earlier steps).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Tuple

import numpy as np


@dataclass
class Hyper:
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.01
    step: int = 1


def adamw_step(theta: np.ndarray, grad: np.ndarray, m: np.ndarray, v: np.ndarray, hp: Hyper
               ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """One AdamW step in fp64; returns (theta, m, v) as new arrays."""
    theta = np.asarray(theta, dtype=np.float64)
    g = np.asarray(grad, dtype=np.float64)
    m = hp.beta1 * np.asarray(m, dtype=np.float64) + (1.0 - hp.beta1) * g
    v = hp.beta2 * np.asarray(v, dtype=np.float64) + (1.0 - hp.beta2) * g * g
    mh = m / (1.0 - hp.beta1 ** hp.step)
    vh = v / (1.0 - hp.beta2 ** hp.step)
    theta = theta - hp.lr * (mh / (np.sqrt(vh) + hp.eps) + hp.weight_decay * theta)
    return theta, m, v
