"""Host-side integers of the grow-then-evict cycle (Sec. 4.1 of the paper).

The kernels take an explicit keep count per segment; this module turns a
retention rate and a cadence into those counts.

Two rules are offered because the paper and the benchmark configurations read
differently: the paper keeps a fixed *fraction* of the current cache every
round (whose steady state before a round is delta / eps, Appendix A.2); the
benchmark configurations fix a *budget* (a fraction of the initial cache) and
every round evicts down to it.
"""
from __future__ import annotations

from typing import List

import numpy as np


def keep_count(n: int, num: int, den: int) -> int:
    """ceil(n * num / den) in exact integer arithmetic, clamped to [1, n] (0 for an empty segment)."""
    if n <= 0:
        return 0
    return max(1, min(n, (n * num + den - 1) // den))


def keep_counts(n: np.ndarray, num: int, den: int) -> np.ndarray:
    n = np.asarray(n, dtype=np.int64)
    k = (n * num + den - 1) // den
    return np.where(n <= 0, 0, np.clip(k, 1, np.maximum(n, 1))).astype(np.int32)


def split_budget(total: int, weights: np.ndarray, n_per_head: np.ndarray) -> np.ndarray:
    """Split a sequence's retention budget over its KV heads in proportion to
    `weights` (largest-remainder rounding), never above a head's own length and
    at least 1 per non-empty head.  The shares sum to `total` when the caps allow."""
    w = np.asarray(weights, dtype=np.float64)
    cap = np.asarray(n_per_head, dtype=np.int64)
    raw = total * w / w.sum()
    base = np.floor(raw).astype(np.int64)
    rest = int(total - base.sum())
    order = np.argsort(-(raw - base), kind="stable")
    base[order[:rest]] += 1
    base = np.minimum(np.maximum(base, np.minimum(1, cap)), cap)
    return base.astype(np.int32)


def trajectory(c0: int, delta: int, num: int, den: int, rounds: int, rule: str = "fraction",
               budget: int | None = None) -> List[int]:
    """Cache rows immediately before each of `rounds` eviction rounds."""
    sizes, c = [], c0
    for _ in range(rounds):
        sizes.append(c)
        if rule == "fraction":
            c = keep_count(c, num, den) + delta
        elif rule == "budget":
            b = budget if budget is not None else keep_count(c0, num, den)
            c = min(c, b) + delta
        else:
            raise ValueError(rule)
    return sizes


def peak_reduction(prompt: int, completion: int, delta: int, num: int, den: int) -> float:
    """Peak rows without eviction over peak rows with the fraction rule (the
    memory-saving figure of Sec. 5.1, for one sequence)."""
    total = prompt + completion
    c, peak, t = min(total, delta), 0, min(total, delta)
    peak = c
    while t < total:
        c = keep_count(c, num, den)
        step = min(delta, total - t)
        c += step
        t += step
        peak = max(peak, c)
    return total / peak
