"""Computation-cost model of the paper (Sec. 4.1.2 "Cost Estimation", Eq. 12) for one GPU's share:

    T_comp = alpha1 * sum_k s_k^2 + alpha2 * sum_k s_k + beta1

(the 1/d_p of Eq. 12 is folded into the coefficients: they are fitted for the heads one GPU holds).
The paper obtains alpha1, alpha2, beta1 "through profiling" and reports an estimation error below
6 % (below 5 % in its appendix on estimation accuracy).  `fit` is that profiling step for this
library's attention kernels: an ordinary least-squares fit of measured times, weighted by 1/time so
that it is the RELATIVE error that is minimised.  No attention arithmetic here.
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np


def features(lens: Sequence[int]) -> np.ndarray:
    s = np.asarray(lens, dtype=np.float64)
    return np.array([float((s * s).sum()), float(s.sum()), 1.0])


def fit(batches: Sequence[Sequence[int]], times: Sequence[float]) -> Tuple[float, float, float]:
    """(alpha1, alpha2, beta1) minimising sum(((predicted - measured) / measured)^2)."""
    X = np.stack([features(b) for b in batches])
    y = np.asarray(times, dtype=np.float64)
    if len(y) < 3 or (y <= 0).any():
        raise ValueError("need at least 3 positive measurements")
    w = 1.0 / y
    coef, *_ = np.linalg.lstsq(X * w[:, None], y * w, rcond=None)
    return float(coef[0]), float(coef[1]), float(coef[2])


def predict(coef: Tuple[float, float, float], lens: Sequence[int]) -> float:
    return float(np.dot(np.asarray(coef, dtype=np.float64), features(lens)))


def relative_errors(coef, batches, times) -> np.ndarray:
    y = np.asarray(times, dtype=np.float64)
    return np.array([predict(coef, b) for b in batches]) / y - 1.0
