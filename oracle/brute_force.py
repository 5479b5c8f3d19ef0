"""Dependency-free brute force for tiny T (test infrastructure, not product).

Enumerates every one of the 2^T keep/drop patterns of a head and selects those
that satisfy the per-token rule of Algorithm 1 (Sec. 3.3) read token by token:
a position is kept if and only if it lies among the last `window` positions or
its score is not below tau.  Exactly one pattern can satisfy it; the numpy
oracle must produce that pattern.  Pure Python, no numpy, so it cannot share a
mistake with a vectorised expression.
"""
from __future__ import annotations

from typing import List, Sequence


def consistent_masks(scores: Sequence[float], tau: float, window: int) -> List[List[bool]]:
    T = len(scores)
    found = []
    for code in range(1 << T):
        pattern = [(code >> t) & 1 == 1 for t in range(T)]
        ok = True
        for t in range(T):
            distance_from_end = T - 1 - t          # 0 for the newest token
            protected = distance_from_end < window
            passes = scores[t] >= tau
            should_keep = protected or passes
            if pattern[t] != should_keep:
                ok = False
                break
        if ok:
            found.append(pattern)
    return found


def gather_loop(rows: Sequence[Sequence[int]], pattern: Sequence[bool]) -> List[List[int]]:
    out = []
    for t, kept in enumerate(pattern):
        if kept:
            out.append(list(rows[t]))
    return out
