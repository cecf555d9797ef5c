"""Host-side learning-rate tables for the baselines AdaScale is compared with (Sec. 4 and the
warm-up paragraph of App. B): linear scaling with warm-up, LSW, and its stretched form, LSW+.

Nothing here runs on the device or belongs to the AdaScale step; the tables are what a caller
would hand to a scale-1 context (whose gain is 1 and whose clock is the iteration count) together
with the mean of the S gradients, to train the comparison run through the same library.
"""
from __future__ import annotations

import math
from typing import Sequence

import numpy as np

WARMUP_FRACTION = 0.055   # share of the iterations spent in warm-up (Sec. 4)


def lsw_schedule(lr_table: Sequence[float], S: int, warmup_fraction: float = WARMUP_FRACTION) -> np.ndarray:
    """Linear scaling with warm-up for scale S (Definition 2 of Sec. 3.1 plus the warm-up of Sec. 4).

    The run lasts ceil(T / S) iterations, T = len(lr_table).  Over the first W = round(fraction *
    ceil(T / S)) of them the rate rises linearly from lr(0) to S * lr(0); from W on it is the
    linearly scaled single-batch schedule S * lr(S t), whose first W entries the warm-up replaces
    (the step-decay form of App. B: the total stays ceil(T / S)).
    """
    lr = np.asarray(lr_table, dtype=np.float64)
    if lr.ndim != 1 or lr.size < 1:
        raise ValueError("lr_table must be a non-empty vector")
    if S < 1:
        raise ValueError("S must be >= 1")
    if not 0.0 <= warmup_fraction < 1.0:
        raise ValueError("warmup_fraction must be in [0, 1)")
    T = lr.size
    T_S = math.ceil(T / S)
    W = int(round(warmup_fraction * T_S))
    t = np.arange(T_S)
    out = S * lr[np.minimum(S * t, T - 1)]
    if W > 0:
        out[:W] = lr[0] + (S - 1) * lr[0] * (t[:W] / W)
    return out.astype(np.float32)


def lsw_plus_schedule(lr_table: Sequence[float], S: int, iterations: int,
                      warmup_fraction: float = WARMUP_FRACTION) -> np.ndarray:
    """LSW+ (Sec. 4): the LSW schedule stretched along the iteration axis to `iterations` steps
    (the number AdaScale took at the same scale), entry t taken from LSW's entry floor(t * T_S / iterations)."""
    if iterations < 1:
        raise ValueError("iterations must be >= 1")
    base = lsw_schedule(lr_table, S, warmup_fraction)
    idx = np.minimum((np.arange(iterations) * base.size) // iterations, base.size - 1)
    return base[idx]
