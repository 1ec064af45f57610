"""The bookkeeping of train() in the asynchronous loop: per-shard learning-rate schedule
(Eq. lr) and data-shard sampling (Eq. data_sample).  Host-side arithmetic in float64.

Readings: the cosine phase uses ratio = (t - t_warmup) / max(T - t_warmup, 0) clamped to
[0, 1], with ratio = 1 when that denominator is 0 (the section on Learning Rate Scheduling asks
for a non-negative denominator and a ratio inside [0, 1]); before any data point has been
learned the progress share n_i / sum n_j counts as 0; if every shard is exactly on target
(all differences <= 0) the size shares themselves are used.
"""
from __future__ import annotations

import math
import numpy as np


def lr_schedule(t, t_warmup, T, eta_max, eta_min):
    """Eq. (lr) for one step index t (0-based count of steps already taken on the shard)."""
    if t < t_warmup:
        return t * eta_max / t_warmup
    denom = max(T - t_warmup, 0)
    ratio = 1.0 if denom == 0 else min(max((t - t_warmup) / denom, 0.0), 1.0)
    return eta_min + 0.5 * (eta_max - eta_min) * (1.0 + math.cos(ratio * math.pi))


def shard_probabilities(sizes, learned):
    """Eq. (data_sample): p_i proportional to max(|D_i| / sum |D_j| - n_i / sum n_j, 0)."""
    sizes = np.asarray(sizes, dtype=np.float64)
    learned = np.asarray(learned, dtype=np.float64)
    if sizes.ndim != 1 or sizes.size == 0 or sizes.shape != learned.shape or np.any(sizes <= 0) or np.any(learned < 0):
        raise ValueError("sizes must be positive, learned non-negative, same length")
    share = sizes / sizes.sum()
    total = learned.sum()
    progress = learned / total if total > 0 else np.zeros_like(learned)
    w = np.maximum(share - progress, 0.0)
    if w.sum() <= 0.0:
        w = share
    return w / w.sum()


def shard_sample(sizes, learned, u):
    """Index drawn from shard_probabilities by inverse CDF with the uniform number u in [0, 1)."""
    p = shard_probabilities(sizes, learned)
    c = 0.0
    for i, pi in enumerate(p):
        c += pi
        if u < c:
            return i
    return int(np.flatnonzero(p > 0)[-1])
