"""Checker for the memory pool of a chain of operators.  TEST INFRASTRUCTURE ONLY.

Section 3.2 ("preparation-execution decoupling"): the memory a whole graph needs is found by walking its
operators without running them and adding up what is taken and given back.  Many placements are correct, so
this module does not compute "the" answer; it states what every correct answer satisfies:

  * ``peak_live``      the largest sum of sizes alive at one operator -- no pool can be smaller;
  * ``violations``     pairs of buffers that are alive at the same operator and overlap in memory
                       (none allowed), plus misaligned or out-of-pool placements;
  * ``walk_high_water`` the literal walk with the simplest possible pool (a bump pointer that is reset
                       whenever nothing is alive): an upper bound any sensible planner must not exceed.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple


def _aligned(b: int, align: int) -> int:
    return (b + align - 1) // align * align


def peak_live(sizes: Sequence[int], first: Sequence[int], last: Sequence[int], align: int = 1) -> int:
    ops = max(last, default=-1) + 1
    best = 0
    for t in range(ops):
        live = sum(_aligned(s, align) for s, f, l in zip(sizes, first, last) if f <= t <= l)
        best = max(best, live)
    return best


def violations(sizes, first, last, offsets, total, align: int = 1) -> List[Tuple[str, int, int]]:
    bad = []
    n = len(sizes)
    for i in range(n):
        if sizes[i] == 0:
            continue
        if offsets[i] % align:
            bad.append(("misaligned", i, i))
        if offsets[i] < 0 or offsets[i] + sizes[i] > total:
            bad.append(("outside", i, i))
    for i in range(n):
        for j in range(i + 1, n):
            if sizes[i] == 0 or sizes[j] == 0:
                continue
            together = first[i] <= last[j] and first[j] <= last[i]
            overlap = offsets[i] < offsets[j] + sizes[j] and offsets[j] < offsets[i] + sizes[i]
            if together and overlap:
                bad.append(("overlap", i, j))
    return bad


def walk_high_water(sizes, first, last, align: int = 1) -> int:
    ops = max(last, default=-1) + 1
    top = 0
    high = 0
    for t in range(ops):
        if not any(f < t <= l for f, l in zip(first, last)):   # nothing carried over from before t
            top = 0
        for s, f in zip(sizes, first):
            if f == t:
                top += _aligned(s, align)
        high = max(high, top)
    return high
