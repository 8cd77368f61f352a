"""Workload partition of arXiv 1712.02546, Section 3.1.1, Eq. (1) -- TEST INFRASTRUCTURE.

Exact rational arithmetic (``fractions.Fraction``), no code shared with the library.
Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may use it.

What the paper fixes (Section 3.1.1): every device times the same probe workload
(``t_i``); its performance value is ``max(t)/t_i`` and its share of the kernels is that
value over the sum of all values (Eq. (1)).  A device that needs ``t_i`` for the whole
workload needs ``w_i * t_i`` for its share.

What the paper leaves open and this file decides: how fractional kernel counts become
integers.  Largest remainder: every device first gets ``floor(w_i * K)`` kernels, the
kernels left over go one each to the devices with the largest fractional parts, equal
fractions to the lower device index first.  Blocks are contiguous and in device order.
"""
from __future__ import annotations

from fractions import Fraction
from typing import List, Sequence


def _exact(t: Sequence) -> List[Fraction]:
    out = [Fraction(v) for v in t]          # a float converts to its exact binary value
    if not out or any(v <= 0 for v in out):
        raise ValueError("times must be positive")
    return out


def performance(t: Sequence) -> List[Fraction]:
    """max(t) / t_i, the numerator of Eq. (1)."""
    tt = _exact(t)
    return [max(tt) / v for v in tt]


def shares(t: Sequence) -> List[Fraction]:
    """w_i of Eq. (1)."""
    perf = performance(t)
    total = sum(perf)
    return [p / total for p in perf]


def kernel_counts(t: Sequence, K: int) -> List[int]:
    """Integer kernel counts that sum to K (largest remainder, see the module header)."""
    if K < 0:
        raise ValueError("K must be non-negative")
    quota = [w * K for w in shares(t)]
    counts = [q.numerator // q.denominator for q in quota]
    frac = [q - c for q, c in zip(quota, counts)]
    left = K - sum(counts)
    order = sorted(range(len(counts)), key=lambda i: (-frac[i], i))
    for i in order[:left]:
        counts[i] += 1
    return counts


def bounds(t: Sequence, K: int) -> List[int]:
    """k-boundaries b[0]=0 <= ... <= b[n]=K; device i owns kernels [b[i], b[i+1])."""
    b = [0]
    for c in kernel_counts(t, K):
        b.append(b[-1] + c)
    return b


def finish_times(t: Sequence, w: Sequence) -> List[Fraction]:
    """Time each device needs for its share w_i of a workload it would finish alone in t_i."""
    return [Fraction(a) * Fraction(b) for a, b in zip(t, w)]


def speedup(t: Sequence, w: Sequence) -> Fraction:
    """Fastest device working alone against the slowest device of the partition
    (the comparison the worked example of Section 3.1.1 makes; communication excluded)."""
    return min(_exact(t)) / max(finish_times(t, w))
