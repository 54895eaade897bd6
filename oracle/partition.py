"""Minimax layer partition by exhaustive search (CPU oracle for Alg. 1, Sec. 4.2).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Definition (Eq. 2): among all ways to cut layers 0..L-1 into P non-empty contiguous blocks, one
per pipeline stage in order, such that every block's memory Mem[a..b] fits its stage's cap, find
one whose largest per-stage mini-step time t_p([a..b]) is smallest.  The paper's dynamic programme
(Eq. 3) reaches exactly this optimum; here every partition is simply tried.
"""
from __future__ import annotations

import itertools
import math


def best_partition(L: int, P: int, t, mem, cap):
    """t[p][a][b], mem[a][b] for 0 <= a <= b < L; cap[p].  Returns (cost, boundaries) with
    boundaries = number of layers in stages 0..p for p = 0..P-2, or (inf, None) if infeasible."""
    best, arg = math.inf, None
    for cuts in itertools.combinations(range(1, L), P - 1):
        edges = (0,) + cuts + (L,)
        worst, ok = 0.0, True
        for p in range(P):
            a, b = edges[p], edges[p + 1] - 1
            if mem[a][b] > cap[p]:
                ok = False
                break
            worst = max(worst, t[p][a][b])
        if ok and worst < best:
            best, arg = worst, list(cuts)
    return best, arg


def partition_cost(L: int, P: int, t, mem, cap, bounds):
    """Worst stage time of a given partition, inf if it violates a cap or is malformed."""
    edges = [0] + list(bounds) + [L]
    if len(edges) != P + 1 or any(edges[i] >= edges[i + 1] for i in range(P)):
        return math.inf
    worst = 0.0
    for p in range(P):
        a, b = edges[p], edges[p + 1] - 1
        if mem[a][b] > cap[p]:
            return math.inf
        worst = max(worst, t[p][a][b])
    return worst
