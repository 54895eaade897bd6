"""Minimax layer partition (Alg. 1, Sec. 4.2): the library's dynamic programme against exhaustive
search (oracle/partition.py), closed forms, and the oracle's own pins.  CPU only."""
import itertools
import math

import numpy as np
import pytest

import paper_2510_00606_amd as ew
from oracle import partition


def tables(L, P, layer_time, layer_mem, stage_speed=None, extra=None):
    """t_p([a..b]) = sum of layer times / stage speed (+ extra[p]); Mem = sum of layer memories."""
    stage_speed = stage_speed or [1.0] * P
    extra = extra or [0.0] * P
    t = np.zeros((P, L, L))
    mem = np.zeros((L, L))
    for a in range(L):
        for b in range(a, L):
            mem[a, b] = sum(layer_mem[a:b + 1])
            for p in range(P):
                t[p, a, b] = sum(layer_time[a:b + 1]) / stage_speed[p] + extra[p]
    return t, mem


def test_oracle_closed_forms():
    # equal layers, equal stages, P | L: the even split with cost L/P; a loose cap changes nothing
    for L, P in ((8, 4), (12, 3), (6, 6), (5, 1)):
        t, mem = tables(L, P, [1.0] * L, [1.0] * L)
        cost, b = partition.best_partition(L, P, t, mem, [L] * P)
        assert cost == L / P and b == [(p + 1) * L // P for p in range(P - 1)]
    # one heavy layer dominates: optimum = its own time when it can sit alone
    t, mem = tables(6, 3, [1, 1, 10, 1, 1, 1], [1] * 6)
    cost, b = partition.best_partition(6, 3, t, mem, [6] * 3)
    assert cost == 10.0 and partition.partition_cost(6, 3, t, mem, [6] * 3, b) == 10.0
    # unequal stages: stage 1 at half speed, four unit layers: (1,3) costs 6, (2,2) 4, (3,1) 3
    t, mem = tables(4, 2, [1.0] * 4, [1.0] * 4, stage_speed=[1.0, 0.5])
    assert partition.best_partition(4, 2, t, mem, [4, 4]) == (3.0, [3])
    # ... and with stage 0 capped at two layers the best left is (2,2)
    assert partition.best_partition(4, 2, t, mem, [2, 4]) == (4.0, [2])
    # a cap of one layer per stage with more layers than stages: infeasible
    t, mem = tables(5, 3, [1] * 5, [1] * 5)
    assert partition.best_partition(5, 3, t, mem, [1, 1, 1]) == (math.inf, None)
    # number of candidates = C(L-1, P-1)
    assert sum(1 for _ in itertools.combinations(range(1, 9), 3)) == math.comb(8, 3)


def check(L, P, t, mem, cap):
    want, wb = partition.best_partition(L, P, t, mem, cap)
    if want == math.inf:
        with pytest.raises(ew.EwError) as e:
            ew.ew_partition_layers(t, mem, cap)
        assert e.value.code == ew.EW_EINFEASIBLE
        return
    cost, bounds = ew.ew_partition_layers(t, mem, cap)
    assert cost == want                                      # the optimum is unique ...
    assert partition.partition_cost(L, P, t, mem, cap, bounds) == want   # ... the partition need not be


def test_against_exhaustive_search():
    rng = np.random.default_rng(0)
    n = 0
    for L in range(1, 10):
        for P in range(1, L + 1):
            for trial in range(6):
                lt = rng.integers(1, 20, L).astype(float)
                lm = rng.integers(1, 10, L).astype(float)
                speed = rng.choice([0.5, 1.0, 2.0], P).tolist()
                t, mem = tables(L, P, lt, lm, speed, rng.integers(0, 3, P).astype(float).tolist())
                total = lm.sum()
                for cap in ([total] * P, [total / P * 1.6] * P, rng.integers(3, 25, P).astype(float).tolist()):
                    check(L, P, t, mem, cap)
                    n += 1
    assert n > 700
    # arbitrary (non-additive) cost tables
    for trial in range(40):
        L, P = int(rng.integers(2, 9)), int(rng.integers(1, 5))
        P = min(P, L)
        t = rng.random((P, L, L))
        mem = rng.random((L, L))
        check(L, P, t, mem, rng.random(P) + 0.3)


def test_slow_stage_gets_fewer_layers():
    # a stage that lost a rank runs its layers slower (larger micro-batch per rank): the partition
    # moves layers away from it, which is what triggers a layer migration
    L, P = 32, 4
    t, mem = tables(L, P, [1.0] * L, [1.0] * L, stage_speed=[1.0, 0.5, 1.0, 1.0])
    cost, b = ew.ew_partition_layers(t, mem, [L] * P)
    sizes = np.diff([0] + b + [L]).tolist()
    assert sizes[1] < min(sizes[0], sizes[2], sizes[3])
    assert cost == max(sizes[0], 2 * sizes[1], sizes[2], sizes[3])
    assert cost < 2 * (L // P)        # better than keeping the even split


def test_partition_errors():
    t, mem = tables(4, 2, [1] * 4, [1] * 4)
    with pytest.raises(ew.EwError) as e:
        ew.ew_partition_layers(np.zeros((5, 4, 4)), mem, [1] * 5)   # more stages than layers
    assert e.value.code == ew.EW_EINVAL
    with pytest.raises(ValueError):
        ew.ew_partition_layers(t, mem, [1.0])
    assert "infeasible" in ew.ew_strerror(ew.EW_EINFEASIBLE)
