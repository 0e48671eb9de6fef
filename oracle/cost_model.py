"""Oracle: the linear compute-time model of one partition, t = a * blocks + c * items + t0.

TEST INFRASTRUCTURE ONLY (see the package docstring).

What is followed: the paper's latency model takes the attention time of one GPU as a term
proportional to the dense-block count plus a constant launch term, with constants fitted offline
from profiles (Methodology, "Sparsity-aware Strategy Selection", the L_comp term of the latency
equation).  On one GPU the unit that runs alone is a partition (one persistent workgroup); it
also pays a fixed cost per work item (loading the query tile, storing the result), so the model
has one more term.  The fit is ordinary least squares, written as the library call that defines
it (numpy.linalg.lstsq on the design matrix [blocks, items, 1]).

Readings: the paper does not print its fitting procedure; least squares on per-partition
samples is this build's choice.  A rank-deficient design (e.g. items proportional to blocks in
every sample) has no unique fit and is an error.
"""

from __future__ import annotations

import numpy as np


def fit(blocks, items, time):
    """Returns (a, c, t0, rms residual).  Raises ValueError when the samples do not determine the model."""
    X = np.stack([np.asarray(blocks, dtype=np.float64), np.asarray(items, dtype=np.float64),
                  np.ones(len(blocks), dtype=np.float64)], axis=1)
    y = np.asarray(time, dtype=np.float64)
    if X.shape[0] < 3 or np.linalg.matrix_rank(X) < 3:
        raise ValueError("samples do not determine the three constants")
    coef, *_ = np.linalg.lstsq(X, y, rcond=None)
    r = y - X @ coef
    return float(coef[0]), float(coef[1]), float(coef[2]), float(np.sqrt(np.mean(r * r)))


def predict(blocks, items, a: float, c: float, t0: float):
    """Model time of each partition; the kernel ends with the slowest one."""
    return [a * float(b) + c * float(i) + t0 for b, i in zip(blocks, items)]
