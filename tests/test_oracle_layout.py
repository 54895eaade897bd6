"""Pins for oracle/layout.py and oracle/brute.py (CPU only).

Each test checks the oracle against something that is not the oracle: the
paper's D=4, F={2} scenario (tests/golden/live_remap_d4_f2.txt), closed forms,
numpy library routines in special cases, or per-element brute force.
"""
import itertools
import os

import numpy as np
import pytest

from oracle import brute, layout

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "live_remap_d4_f2.txt")


def recoverable_masks(old_dp):
    out = []
    for m in range(1, 1 << old_dp):
        alive = [(m >> j) & 1 for j in range(old_dp)]
        if all(alive[j] or alive[(j - 1) % old_dp] for j in range(old_dp)):
            out.append(m)
    return out


def make_state(starts, old_dp, alive, rng, dtype=np.int64, poison=None):
    """Old shards and snapshots with distinct values everywhere."""
    lens = layout.shard_lengths(starts, old_dp)
    shards, snaps = [], []
    for j in range(old_dp):
        v = rng.integers(0, 1 << 40, size=lens[j]).astype(dtype)
        if alive[j]:
            shards.append(v)
            snaps.append(None)
        else:
            shards.append(None if poison is None else np.full(lens[j], poison, dtype))
            snaps.append(v)
    return shards, snaps


# --------------------------------------------------------------- P1: paper's scenario
def read_golden():
    rows = {"A": [], "B": [], "S": []}
    with open(GOLDEN) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            t = line.split()
            rows[t[0]].append(t[1:])
    return rows


def labelled_cells(old_dp, new_dp, mask, starts):
    """Run the oracle on label data; return {(owner, kind, new_rank): count}."""
    alive = layout.alive_list(old_dp, mask)
    lens = layout.shard_lengths(starts, old_dp)
    shards = [np.full(lens[j], 10 * j + 1, np.int32) for j in range(old_dp)]
    snaps = [np.full(lens[j], 10 * j + 2, np.int32) for j in range(old_dp)]
    for j in range(old_dp):
        if not alive[j]:
            shards[j] = np.full(lens[j], 99, np.int32)  # a dead device: must never be read
    new = layout.reshard(shards, snaps, old_dp, new_dp, mask, starts)
    cells = {}
    for k, sh in enumerate(new):
        vals, cnt = np.unique(sh, return_counts=True)
        for v, c in zip(vals, cnt):
            cells[(int(v) // 10, {1: "live", 2: "snap", 9: "dead"}[int(v) % 10], k)] = int(c)
    return cells, new


def test_paper_scenario_d4_f2():
    g = read_golden()
    starts = layout.unit_starts(1 << 20, 4096)
    mask = 0b1011
    cells, new = labelled_cells(4, 3, mask, starts)
    assert not any(kind == "dead" for (_, kind, _) in cells)
    alive = layout.alive_list(4, mask)
    nro = layout.new_rank_of(4, 3, alive)
    assert nro == [0, 1, -1, 2]
    # Part A: pairs the captions print
    for owner, kind, holder, dst_old, dst_new, loc in g["A"]:
        owner, holder, dst_old, dst_new = map(int, (owner, holder, dst_old, dst_new))
        assert (owner, kind, dst_new) in cells
        assert layout.holder_of(owner, 4, alive) == holder
        assert nro[dst_old] == dst_new and nro[holder] != dst_new
    # Part B: complete cell set with per-unit element counts
    want = {}
    for owner, kind, holder, dst_old, dst_new, loc, n in g["B"]:
        want[(int(owner), kind, int(dst_new))] = int(n) * 256
        assert (nro[int(holder)] == int(dst_new)) == (loc == "local")
    assert cells == want
    assert [len(s) for s in new] == [int(x) for x in g["S"][0]]
    # the same cells, seen as messages in the staging arena
    lens = layout.shard_lengths(starts, 4)
    sh = [np.arange(lens[j], dtype=np.int64) + (j << 32) for j in range(4)]
    arena, table = layout.staging(sh[:2] + [None] + sh[3:], [None, None, sh[2], None], 4, 3, mask, starts)
    assert set(table) == {(1, 0), (1, 2)}
    assert table[(1, 0)] == (0, 336 * 256) and table[(1, 2)] == (336 * 256, 344 * 256)
    assert (arena[:336 * 256] >> 32 == 1).all() and (arena[336 * 256:] >> 32 == 2).all()


def test_snapshot_holder_is_ring_predecessor():
    # worker i backs up worker (i+1) mod n  (Sec. 5.1)
    for n in range(2, 9):
        for f in range(n):
            alive = [j != f for j in range(n)]
            assert layout.holder_of(f, n, alive) == (f - 1) % n
            for j in range(n):
                if j != f:
                    assert layout.holder_of(j, n, alive) == j
    with pytest.raises(layout.Unrecoverable):
        layout.check_recoverable(4, [True, False, False, True])
    with pytest.raises(layout.Unrecoverable):
        layout.check_recoverable(1, [False])
    with pytest.raises(layout.Unrecoverable):
        layout.check_recoverable(3, [False, False, False])
    layout.check_recoverable(4, [False, True, False, True])


# --------------------------------------------------------------- layout definition
def test_piece_bounds_properties():
    for L in list(range(0, 70)) + [100, 1000, 4096, 4099, 262144, 65536]:
        for D in range(1, 18):
            b = layout.piece_bounds(L, D)
            assert b[0] == 0 and b[-1] == L and len(b) == D + 1
            assert all(b[i] <= b[i + 1] for i in range(D))
            assert all(x % 8 == 0 for x in b[:-1])
            sizes = [b[i + 1] - b[i] for i in range(D)]
            # uniform: pieces differ by at most one granule
            assert max(sizes) - min(sizes) <= 8
            if L % (8 * D) == 0:
                assert sizes == [L // D] * D


def test_every_rank_owns_a_piece_of_every_unit():
    # Fig. 10b: rank j owns the j-th shard of every layer
    starts = layout.unit_starts(10 * 4096 + 520, 4096)
    for D in (2, 3, 5, 8):
        emap, _ = brute.element_map(starts, D)
        seen = {(u, j) for (u, j, _) in emap}
        assert seen == {(u, j) for u in range(len(starts) - 1) for j in range(D)}


# --------------------------------------------------------------- P2: closed form D -> D+1
@pytest.mark.parametrize("D", [1, 2, 3, 4, 5, 7])
def test_scale_up_local_fraction_is_half(D):
    L = 8 * D * (D + 1) * 3
    starts = layout.unit_starts(5 * L, L)
    mask = (1 << D) - 1
    cells, _ = labelled_cells(D, D + 1, mask, starts)
    N = 5 * L
    local = sum(c for (owner, kind, k), c in cells.items() if owner == k)
    assert 2 * local == N
    for j in range(D):
        # overlap of [j/D,(j+1)/D) with [j/(D+1),(j+1)/(D+1)) is (D-j)/(D(D+1))
        assert cells.get((j, "live", j), 0) * D * (D + 1) == (D - j) * N
    assert all(kind == "live" for (_, kind, _) in cells)


# --------------------------------------------------------------- P4: library special cases
def test_identity_when_nothing_changes():
    rng = np.random.default_rng(1)
    starts = layout.unit_starts(4099, 100)
    for D in (1, 3, 6):
        alive = [True] * D
        sh, sn = make_state(starts, D, alive, rng)
        new = layout.reshard(sh, sn, D, D, (1 << D) - 1, starts)
        for a, b in zip(sh, new):
            assert a.tobytes() == b.tobytes()
        arena, table = layout.staging(sh, sn, D, D, (1 << D) - 1, starts)
        assert len(arena) == 0 and not table


def test_single_unit_is_numpy_split():
    rng = np.random.default_rng(2)
    for Do, Dn in itertools.product((1, 2, 3, 4, 6), repeat=2):
        N = 8 * 12 * 5 * 7
        flat = rng.integers(0, 1 << 50, N)
        starts = layout.unit_starts(N, N)
        old = np.split(flat, Do)
        new = layout.reshard(old, [None] * Do, Do, Dn, (1 << Do) - 1, starts)
        for a, b in zip(new, np.split(flat, Dn)):
            assert np.array_equal(a, b)


def test_gather_and_scatter_extremes():
    rng = np.random.default_rng(3)
    starts = layout.unit_starts(1000, 24)
    for D in (2, 5):
        sh, sn = make_state(starts, D, [True] * D, rng)
        flat = layout.reconstruct_flat(sh, sn, D, [True] * D, starts)
        # Dn = 1: the one new shard is the flat state
        (one,) = layout.reshard(sh, sn, D, 1, (1 << D) - 1, starts)
        assert np.array_equal(one, flat)
        # Do = 1: pure scatter; gathering back restores it
        parts = layout.reshard([flat], [None], 1, D, 1, starts)
        for a, b in zip(parts, sh):
            assert np.array_equal(a, b)


def test_round_trip_restores_old_shards():
    rng = np.random.default_rng(4)
    for (Do, Dn, N, C) in [(4, 3, 4099, 100), (8, 7, 10000, 264), (5, 9, 777, 8), (3, 2, 64, 1)]:
        starts = layout.unit_starts(N, C)
        sh, sn = make_state(starts, Do, [True] * Do, rng)
        mid = layout.reshard(sh, sn, Do, Dn, (1 << Do) - 1, starts)
        back = layout.reshard(mid, [None] * Dn, Dn, Do, (1 << Dn) - 1, starts)
        for a, b in zip(sh, back):
            assert np.array_equal(a, b)
        assert sum(len(x) for x in mid) == N


# --------------------------------------------------------------- P6: brute force
def brute_expected(starts, Do, Dn, alive, shards, snaps):
    emap, new_len = brute.reshard_map(starts, Do, Dn, alive)
    new = [np.zeros(n, dtype=np.int64) for n in new_len]
    wrote = [np.zeros(n, dtype=np.int32) for n in new_len]
    for (j, oo, snap, holder, k, no) in emap:
        src = snaps[j] if snap else shards[j]
        new[k][no] = src[oo]
        wrote[k][no] += 1
    assert all((w == 1).all() for w in wrote)  # every element lands exactly once
    return emap, new


def brute_arena(emap, Do, Dn, alive, shards, snaps):
    nro = layout.new_rank_of(Do, Dn, alive)
    out, table, off = [], {}, 0
    for k in range(Dn):
        for h in range(Do):
            vals = [(snaps[j] if snap else shards[j])[oo]
                    for (j, oo, snap, holder, kk, no) in emap
                    if holder == h and kk == k and nro[h] != k]
            if vals:
                table[(h, k)] = (off, len(vals))
                off += len(vals)
                out.extend(vals)
    return np.asarray(out, dtype=np.int64), table


def check_case(Do, Dn, mask, N, C, rng):
    starts = layout.unit_starts(N, C)
    alive = layout.alive_list(Do, mask)
    sh, sn = make_state(starts, Do, alive, rng, poison=-1)
    got = layout.reshard(sh, sn, Do, Dn, mask, starts)
    emap, want = brute_expected(starts, Do, Dn, alive, sh, sn)
    assert len(got) == len(want) == Dn
    for a, b in zip(got, want):
        assert np.array_equal(a, b)
    arena, table = layout.staging(sh, sn, Do, Dn, mask, starts)
    b_arena, b_table = brute_arena(emap, Do, Dn, alive, sh, sn)
    assert table == b_table
    assert np.array_equal(arena, b_arena)
    # one-by-one locator agrees with the scan
    for k in range(Dn):
        n = len(want[k])
        if n == 0:
            continue
        glob, owner, ooff = layout.locate_new_elements(starts, Do, Dn, k, np.arange(n))
        ref = [(e, j, oo) for e, (j, oo, _, _, kk, no) in enumerate(emap) if kk == k]
        assert [tuple(map(int, t)) for t in zip(glob, owner, ooff)] == ref


def test_brute_force_all_small_memberships():
    rng = np.random.default_rng(5)
    n = 0
    for Do in range(1, 6):
        for Dn in range(1, 6):
            for mask in recoverable_masks(Do):
                for N in (0, 1, 7, 8, 9, 64):
                    for C in sorted({1, 8, 24, 100, max(N, 1), N + 1}):
                        check_case(Do, Dn, mask, N, C, rng)
                        n += 1
    assert n > 4000


def test_brute_force_larger_ragged():
    rng = np.random.default_rng(6)
    for Do in range(1, 7):
        masks = recoverable_masks(Do)
        pick = {masks[-1], masks[0], masks[len(masks) // 2]}
        for Dn in range(1, 7):
            for mask in pick:
                for N, C in ((1000, 24), (1000, 100), (4099, 264), (4099, 4099), (4099, 5000)):
                    check_case(Do, Dn, mask, N, C, rng)


# --------------------------------------------------------------- P7: poison
def test_failed_live_shards_are_never_read():
    rng = np.random.default_rng(7)
    starts = layout.unit_starts(4099, 100)
    for mask in (0b101011, 0b010101, 0b111110):
        alive = layout.alive_list(6, mask)
        sh, sn = make_state(starts, 6, alive, rng)
        a = layout.reshard(sh, sn, 6, 4, mask, starts)
        lens = layout.shard_lengths(starts, 6)
        sh2 = [s if alive[j] else np.full(lens[j], -7, np.int64) for j, s in enumerate(sh)]
        b = layout.reshard(sh2, sn, 6, 4, mask, starts)
        for x, y in zip(a, b):
            assert np.array_equal(x, y)
