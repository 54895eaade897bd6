"""Pins for oracle/migrate.py (CPU only): the communication-cost closed forms of Sec. 6.3, the
D one-to-one sends of the interleaved assignment, library special cases, brute force."""
import numpy as np
import pytest

from oracle import layout, migrate
from oracle.migrate import CONTIGUOUS, INTERLEAVED


def stage(n_units, L):
    return np.arange(n_units + 1, dtype=np.int64) * L


def make_shards(starts, D, assignment, rng, tag):
    iv = migrate.rank_intervals(starts, D, assignment)
    return [rng.integers(0, 1 << 40, sum(h - l for l, h in x)) + (tag << 44) for x in iv]


@pytest.mark.parametrize("D", [2, 3, 4, 8])
def test_interleaved_is_D_one_to_one_sends(D):
    # "exactly D 1:1 sends summing to |O_i|", no intra-stage traffic (Sec. 6.3, Communication Cost)
    L = 8 * D * 5
    src, dst = stage(6, L), stage(4, L)
    for n_move in (1, 2, 4):
        m = migrate.traffic(src, dst, D, INTERLEAVED, n_move)
        off = m - np.diag(np.diag(m))
        pairs = {(int(a), int(b)) for a, b in zip(*np.nonzero(off))}
        assert pairs == {(j, D + j) for j in range(D)}
        assert off.sum() == n_move * L
        assert all(off[j, D + j] == n_move * L // D for j in range(D))
        assert migrate.split_traffic(m, D) == (0, n_move * L, 0)


@pytest.mark.parametrize("D", [2, 3, 4, 8])
def test_contiguous_closed_form(D):
    # cross-stage |O_i| plus (D-1)/2 |O_i| of re-compaction in a DP group (Sec. 6.3); here the
    # moved layer is small enough that cut r shifts by r*|O_i|/D without overtaking cut r-1
    L = 8 * D * D * 6
    src, dst = stage(D + 3, L), stage(D + 2, L)
    m = migrate.traffic(src, dst, D, CONTIGUOUS, 1)
    intra_s, cross, intra_d = migrate.split_traffic(m, D)
    assert cross == L
    assert 2 * intra_s == (D - 1) * L
    assert 2 * intra_d == (D - 1) * L
    # the paper's total (D+1)/2 |O_i|: the cross-stage copy plus one group's re-compaction
    assert 2 * (cross + intra_s) == (D + 1) * L
    # versus the interleaved assignment: exactly |O_i|
    assert migrate.split_traffic(migrate.traffic(src, dst, D, INTERLEAVED, 1), D) == (0, L, 0)


def test_contiguous_stage_is_numpy_split():
    rng = np.random.default_rng(0)
    for D in (1, 2, 4, 6):
        starts = stage(5, 8 * 12 * 7)
        flat = rng.integers(0, 1 << 50, int(starts[-1]))
        shards = migrate.scatter(flat, starts, D, CONTIGUOUS)
        for a, b in zip(shards, np.split(flat, D)):
            assert np.array_equal(a, b)
        assert np.array_equal(migrate.gather(shards, starts, D, CONTIGUOUS), flat)


def test_interleaved_stage_matches_layout_module():
    rng = np.random.default_rng(1)
    starts = layout.unit_starts(4099, 264)
    flat = rng.integers(0, 1 << 50, 4099)
    for D in (1, 3, 5):
        a = migrate.scatter(flat, starts, D, INTERLEAVED)
        b = layout.slice_flat(flat, D, starts)
        assert all(np.array_equal(x, y) for x, y in zip(a, b))


@pytest.mark.parametrize("assignment", [INTERLEAVED, CONTIGUOUS])
def test_migration_preserves_the_logical_state(assignment):
    # ownership changes, the two stages' flat arrays only exchange the moved layers
    rng = np.random.default_rng(2)
    for D, src, dst, n_move in ((3, [0, 100, 364, 1000], [0, 264, 500], 2), (4, [0, 8, 16, 4099], [0, 7], 1),
                                (2, [0, 50, 120], [0, 30, 90, 91], 0), (5, [0, 1000], [0, 24, 48], 1)):
        src, dst = np.asarray(src, np.int64), np.asarray(dst, np.int64)
        s_sh = make_shards(src, D, assignment, rng, 1)
        d_sh = make_shards(dst, D, assignment, rng, 2)
        ns, nd = migrate.migrate(s_sh, d_sh, src, dst, D, assignment, n_move)
        new_src, new_dst, cut = migrate.moved_starts(src, dst, n_move)
        fs, fd = migrate.gather(s_sh, src, D, assignment), migrate.gather(d_sh, dst, D, assignment)
        assert np.array_equal(migrate.gather(ns, new_src, D, assignment), fs[:cut])
        assert np.array_equal(migrate.gather(nd, new_dst, D, assignment), np.concatenate([fs[cut:], fd]))
        assert sum(map(len, ns)) + sum(map(len, nd)) == len(fs) + len(fd)
        # moving back restores everything (reverse = move the first units of S+1 to the end of S)
        bs = migrate.gather(nd, new_dst, D, assignment)
        moved_len = int(src[-1]) - cut
        assert np.array_equal(np.concatenate([fs[:cut], bs[:moved_len]]), fs)


def test_interleaved_rank_keeps_piece_j_of_every_layer():
    # after the migration rank j of stage S+1 holds [its pieces of the moved layers] + [its old shard]
    rng = np.random.default_rng(3)
    D, L = 4, 8 * 4 * 9
    src, dst = stage(5, L), stage(3, L)
    s_sh = make_shards(src, D, INTERLEAVED, rng, 1)
    d_sh = make_shards(dst, D, INTERLEAVED, rng, 2)
    ns, nd = migrate.migrate(s_sh, d_sh, src, dst, D, INTERLEAVED, 2)
    per = L // D
    for j in range(D):
        assert np.array_equal(ns[j], s_sh[j][:3 * per])
        assert np.array_equal(nd[j], np.concatenate([s_sh[j][3 * per:], d_sh[j]]))


def test_hand_worked_migration_of_unequal_layers():
    # Stage S holds layers of 16, 24, 32 elements, stage S+1 layers of 8 and 40; D = 2; element i of
    # layer l carries the value 1000*l + i.  Granule floor split of a layer of L elements over 2 ranks:
    # 16 -> 8|8, 24 -> 8|16, 32 -> 16|16, 8 -> 0|8, 40 -> 16|24.  All expected arrays below are written
    # out by hand from those cuts, none comes from the oracle.
    def lay(l, a, b):
        return [1000 * l + i for i in range(a, b)]
    src, dst = np.asarray([0, 16, 40, 72]), np.asarray([0, 8, 48])
    s_sh = [np.asarray(lay(0, 0, 8) + lay(1, 0, 8) + lay(2, 0, 16)), np.asarray(lay(0, 8, 16) + lay(1, 8, 24) + lay(2, 16, 32))]
    d_sh = [np.asarray(lay(4, 0, 16)), np.asarray(lay(3, 0, 8) + lay(4, 16, 40))]
    # the LAST layer of stage S becomes the FIRST layer of stage S+1
    new_src, new_dst, cut = migrate.moved_starts(src, dst, 1)
    assert new_src.tolist() == [0, 16, 40] and new_dst.tolist() == [0, 32, 40, 80] and cut == 40
    ns, nd = migrate.migrate(s_sh, d_sh, src, dst, 2, INTERLEAVED, 1)
    assert ns[0].tolist() == lay(0, 0, 8) + lay(1, 0, 8) and ns[1].tolist() == lay(0, 8, 16) + lay(1, 8, 24)
    assert nd[0].tolist() == lay(2, 0, 16) + lay(4, 0, 16)
    assert nd[1].tolist() == lay(2, 16, 32) + lay(3, 0, 8) + lay(4, 16, 40)
    # two layers move: they keep their order in front of stage S+1's own layers
    new_src, new_dst, cut = migrate.moved_starts(src, dst, 2)
    assert new_src.tolist() == [0, 16] and new_dst.tolist() == [0, 24, 56, 64, 104] and cut == 16
    ns, nd = migrate.migrate(s_sh, d_sh, src, dst, 2, INTERLEAVED, 2)
    assert ns[0].tolist() == lay(0, 0, 8) and ns[1].tolist() == lay(0, 8, 16)
    assert nd[0].tolist() == lay(1, 0, 8) + lay(2, 0, 16) + lay(4, 0, 16)
    assert nd[1].tolist() == lay(1, 8, 24) + lay(2, 16, 32) + lay(3, 0, 8) + lay(4, 16, 40)
    # contiguous rule, one layer moves: a stage's whole array gets one granule floor split, before
    # 72 -> 32|40 and 48 -> 24|24, afterwards 40 -> 16|24 and 80 -> 40|40
    cs = [np.asarray(lay(0, 0, 16) + lay(1, 0, 16)), np.asarray(lay(1, 16, 24) + lay(2, 0, 32))]       # 72 -> 32|40
    cd = [np.asarray(lay(3, 0, 8) + lay(4, 0, 16)), np.asarray(lay(4, 16, 40))]                       # 48 -> 24|24
    ns, nd = migrate.migrate(cs, cd, src, dst, 2, CONTIGUOUS, 1)
    assert ns[0].tolist() == lay(0, 0, 16) and ns[1].tolist() == lay(1, 0, 24)                        # 40 -> 16|24
    assert nd[0].tolist() == lay(2, 0, 32) + lay(3, 0, 8) and nd[1].tolist() == lay(4, 0, 40)         # 80 -> 40|40
