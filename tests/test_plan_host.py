"""Host-side tests (no GPU): the C-ABI library loads and exports what include/elaswave.h
declares; ew_plan's segment table satisfies the invariants of the transfer plan and induces
exactly the oracle's element map; error paths."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2510_00606_amd as ew
from oracle import brute, layout
from paper_2510_00606_amd import binding, configs


def recoverable_masks(old_dp):
    out = []
    for m in range(1, 1 << old_dp):
        alive = [(m >> j) & 1 for j in range(old_dp)]
        if all(alive[j] or alive[(j - 1) % old_dp] for j in range(old_dp)):
            out.append(m)
    return out


# ------------------------------------------------------------------ boundary
def test_library_exports_every_declared_symbol(repo_root):
    hdr = open(os.path.join(repo_root, "include", "elaswave.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(ew_[a-z0-9_]+)\s*\(", hdr))
    assert {"ew_plan", "ew_pack", "ew_unpack", "ew_snapshot", "ew_verify", "ew_plan_bounds"} <= declared
    handle = ctypes.CDLL(binding.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(handle, name), f"{name} declared in elaswave.h but not exported"
    assert declared == set(binding.EXPORTS), "binding and header disagree"
    assert "gfx950" in ew.ew_version()


def test_seg_struct_layout_matches_header():
    assert binding.SEG_DTYPE.itemsize == 40
    assert binding.CKSUM_DTYPE.itemsize == 16


# ------------------------------------------------------------------ errors
def test_error_codes():
    def code(*a):
        with pytest.raises(ew.EwError) as e:
            ew.ew_plan(*a)
        return e.value.code

    assert code(0, 3, 0, 100, 10) == ew.EW_EINVAL
    assert code(4, 0, 0b1111, 100, 10) == ew.EW_EINVAL
    assert code(65, 3, 1, 100, 10) == ew.EW_EINVAL
    assert code(4, 3, 0b1111, 100, 0) == ew.EW_EINVAL
    assert code(4, 3, 0b11111, 100, 10) == ew.EW_EINVAL        # bit above old_dp
    assert code(4, 3, 0, 100, 10) == ew.EW_EUNRECOVERABLE      # no survivor
    assert code(4, 3, 0b1001, 100, 10) == ew.EW_EUNRECOVERABLE  # 1 and 2 failed: 2's holder is 1
    assert code(1, 1, 0, 100, 10) == ew.EW_EUNRECOVERABLE
    with pytest.raises(ew.EwError) as e:
        ew.ew_plan_bounds(2, 2, 3, [0, 10, 5])
    assert e.value.code == ew.EW_EINVAL
    with pytest.raises(ew.EwError) as e:
        ew.ew_plan_bounds(2, 2, 3, [1, 10])
    assert e.value.code == ew.EW_EINVAL
    assert "unrecoverable" in ew.ew_strerror(ew.EW_EUNRECOVERABLE)
    # not uploaded: pack/unpack refuse before touching any buffer
    p = ew.ew_plan(4, 3, 0b1011, 4096, 512)
    with pytest.raises(ew.EwError) as e:
        ew.ew_pack(p, [1, 1, 0, 1], [0, 0, 1, 0], 1, 4)
    assert e.value.code == ew.EW_EINVAL
    with pytest.raises(ew.EwError):
        ew.ew_set_param("no_such_knob", 1)
    with pytest.raises(ew.EwError):
        ew.ew_set_param("cksum_sub_bytes", 3000)
    assert ew.ew_get_param("xcd_group_kib") == 2048 and ew.ew_get_param("no_such_knob") == -1
    for bad in (-1, 9):
        with pytest.raises(ew.EwError):
            ew.ew_set_param("fused_wgs_per_cu", bad)
    ew.ew_set_param("fused_wgs_per_cu", 4)
    assert ew.ew_get_param("fused_wgs_per_cu") == 4
    ew.ew_set_param("fused_wgs_per_cu", 0)


def test_max_degree_and_wide_mask():
    p = ew.ew_plan(64, 63, (1 << 64) - 1 - (1 << 63), 64 * 63 * 8 * 3, 64 * 63 * 8)
    assert p.holder_of(63) == 62 and p.new_rank_of(63) == -1
    assert sum(p.new_shard_len(k) for k in range(63)) == p.numel


# ------------------------------------------------------------------ invariants of the table
def check_invariants(p: ew.Plan, old_dp, new_dp, mask, numel):
    segs = p.segs()
    alive = [(mask >> j) & 1 for j in range(old_dp)]
    nro = [p.new_rank_of(j) for j in range(old_dp)]
    assert int(segs["len"].sum()) == numel == p.numel
    assert (segs["len"] > 0).all()
    old_len = [p.old_shard_len(j) for j in range(old_dp)]
    new_len = [p.new_shard_len(k) for k in range(new_dp)]
    assert sum(old_len) == sum(new_len) == numel
    # membership
    for s in segs:
        j, h, k = int(s["src_owner"]), int(s["holder"]), int(s["dst_rank"])
        assert alive[h]
        assert bool(s["flags"] & ew.EW_SEG_SNAPSHOT) == (not alive[j])
        assert h == (j if alive[j] else (j - 1) % old_dp) == p.holder_of(j)
        assert bool(s["flags"] & ew.EW_SEG_LOCAL) == (nro[h] == k)
        assert (s["stage_off"] == ew.EW_NO_STAGE) == bool(s["flags"] & ew.EW_SEG_LOCAL)
    # segments tile every new shard and every old shard exactly
    for key_rank, key_off, lens in (("dst_rank", "dst_off", new_len), ("src_owner", "src_off", old_len)):
        for r, n in enumerate(lens):
            sel = segs[segs[key_rank] == r]
            order = np.argsort(sel[key_off], kind="stable")
            off, ln = sel[key_off][order].astype(np.int64), sel["len"][order].astype(np.int64)
            assert int(ln.sum()) == n
            if n:
                assert off[0] == 0 and (off[1:] == off[:-1] + ln[:-1]).all()
    # arena: contiguous pair messages sorted by (dst, holder); segments fill each message in order
    rem = segs[(segs["flags"] & ew.EW_SEG_LOCAL) == 0]
    assert int(rem["len"].sum()) == p.stage_len == p.remote_elems
    expect_off = 0
    for k in range(new_dp):
        for h in range(old_dp):
            n = p.pair_len(h, k)
            sel = rem[(rem["holder"] == h) & (rem["dst_rank"] == k)]
            assert int(sel["len"].sum()) == n
            if n:
                assert p.pair_off(h, k) == expect_off
                so, ln = sel["stage_off"].astype(np.int64), sel["len"].astype(np.int64)
                assert so[0] == expect_off and (so[1:] == so[:-1] + ln[:-1]).all()
                expect_off += n
    # balance: shard lengths within one granule per unit of each other is implied by the layout;
    # here: identical to the oracle's lengths (checked by the caller)
    return segs


def induced_map(segs, new_len):
    """(new rank, new offset) -> (owner, old offset, snapshot?, holder, stage position or -1)."""
    out = [[None] * n for n in new_len]
    for s in segs:
        k = int(s["dst_rank"])
        local = bool(s["flags"] & ew.EW_SEG_LOCAL)
        for i in range(int(s["len"])):
            slot = int(s["dst_off"]) + i
            assert out[k][slot] is None, "element written twice"
            out[k][slot] = (int(s["src_owner"]), int(s["src_off"]) + i, bool(s["flags"] & ew.EW_SEG_SNAPSHOT),
                            int(s["holder"]), -1 if local else int(s["stage_off"]) + i)
    assert all(x is not None for row in out for x in row), "element never written"
    return out


def check_against_brute(old_dp, new_dp, mask, numel, chunk):
    p = ew.ew_plan(old_dp, new_dp, mask, numel, chunk)
    starts = layout.unit_starts(numel, chunk)
    assert [p.old_shard_len(j) for j in range(old_dp)] == layout.shard_lengths(starts, old_dp)
    assert [p.new_shard_len(k) for k in range(new_dp)] == layout.shard_lengths(starts, new_dp)
    segs = check_invariants(p, old_dp, new_dp, mask, numel)
    alive = layout.alive_list(old_dp, mask)
    emap, new_len = brute.reshard_map(starts, old_dp, new_dp, alive)
    got = induced_map(segs, new_len)
    nro = layout.new_rank_of(old_dp, new_dp, alive)
    assert [p.new_rank_of(j) for j in range(old_dp)] == nro
    # arena positions by the oracle's rule: pairs sorted by (dst, holder), ascending element order
    pos, cur = {}, 0
    for k in range(new_dp):
        for h in range(old_dp):
            for e, (j, oo, snap, holder, kk, no) in enumerate(emap):
                if holder == h and kk == k and nro[h] != k:
                    pos[e] = cur
                    cur += 1
    for e, (j, oo, snap, holder, k, no) in enumerate(emap):
        assert got[k][no] == (j, oo, snap, holder, pos.get(e, -1))
    # explicit-boundary entry point builds the same table
    q = ew.ew_plan_bounds(old_dp, new_dp, mask, starts)
    assert q.segs().tobytes() == segs.tobytes()


def test_table_equals_brute_force_small():
    n = 0
    for Do in range(1, 6):
        for Dn in range(1, 6):
            for mask in recoverable_masks(Do):
                for N in (0, 1, 7, 8, 9, 64):
                    for C in sorted({1, 8, 24, 100, max(N, 1), N + 1}):
                        check_against_brute(Do, Dn, mask, N, C)
                        n += 1
    assert n > 4000


def test_table_equals_brute_force_ragged():
    for Do in range(1, 7):
        masks = recoverable_masks(Do)
        for Dn in range(1, 7):
            for mask in {masks[-1], masks[0], masks[len(masks) // 2]}:
                for N, C in ((1000, 24), (1000, 100), (4099, 264), (4099, 4099), (4099, 5000)):
                    check_against_brute(Do, Dn, mask, N, C)


def test_paper_scenario_pairs():
    # D = 4, F = {2} (Sec. 5.2, Fig. 7): golden per-unit cells, see tests/golden/live_remap_d4_f2.txt
    rows = [l.split()[1:] for l in open(os.path.join(os.path.dirname(__file__), "golden", "live_remap_d4_f2.txt"))
            if l.startswith("B ")]
    p = ew.ew_plan(4, 3, 0b1011, 1 << 20, 4096)
    segs = p.segs()
    cells = {}
    for s in segs:
        key = (int(s["src_owner"]), "snap" if s["flags"] & ew.EW_SEG_SNAPSHOT else "live", int(s["holder"]),
               int(s["dst_rank"]), "local" if s["flags"] & ew.EW_SEG_LOCAL else "remote")
        cells[key] = cells.get(key, 0) + int(s["len"])
    want = {(int(o), kind, int(h), int(dn), loc): int(n) * 256 for o, kind, h, do, dn, loc, n in rows}
    assert cells == want
    assert p.pair_len(1, 0) == 336 * 256 and p.pair_len(1, 2) == 344 * 256
    assert not (segs["holder"] == 2).any()


@pytest.mark.parametrize("name", ["7b_stage", "13b_stage", "70b_stage"])
def test_full_size_plans_are_consistent(name):
    w = configs.ALL[name]()
    starts = w.unit_starts()
    p = ew.ew_plan_bounds(w.old_dp, w.new_dp, w.alive_mask, starts)
    segs = p.segs()
    assert int(segs["len"].sum()) == w.numel
    nb = layout._bounds_matrix(starts.astype(np.int64), w.new_dp)
    ob = layout._bounds_matrix(starts.astype(np.int64), w.old_dp)
    assert [p.new_shard_len(k) for k in range(w.new_dp)] == (nb[:, 1:] - nb[:, :-1]).sum(axis=0).tolist()
    assert [p.old_shard_len(j) for j in range(w.old_dp)] == (ob[:, 1:] - ob[:, :-1]).sum(axis=0).tolist()
    # every boundary is on the 8-element granule for these shapes: 128-bit aligned everywhere
    for f in ("src_off", "dst_off", "len"):
        assert (segs[f] % 8 == 0).all()
    rem = segs[(segs["flags"] & ew.EW_SEG_LOCAL) == 0]
    assert (rem["stage_off"] % 8 == 0).all()
    # sampled elements of every new shard: table agrees with the oracle's one-by-one locator
    rng = np.random.default_rng(w.seed)
    for k in range(w.new_dp):
        sel = segs[segs["dst_rank"] == k]
        order = np.argsort(sel["dst_off"])
        sel = sel[order]
        offs = np.sort(rng.integers(0, p.new_shard_len(k), 4000))
        glob, owner, ooff = layout.locate_new_elements(starts.astype(np.int64), w.old_dp, w.new_dp, k, offs)
        i = np.searchsorted(sel["dst_off"].astype(np.int64), offs, side="right") - 1
        assert (sel["src_owner"][i] == owner).all()
        assert (sel["src_off"][i].astype(np.int64) + (offs - sel["dst_off"][i].astype(np.int64)) == ooff).all()
    if name == "70b_stage":
        assert abs(p.stage_len / w.numel - 0.5) < 1e-4  # D -> D+1 closed form: half stays local


# ------------------------------------------------------------------ copy tiles (host view of what the kernels decode)
def expand(records):
    """records: (src_buf, src_off, dst_buf, dst_off, len) -> per-element rows sorted by destination."""
    rows = []
    for sb, so, db, do, n in records:
        i = np.arange(int(n), dtype=np.int64)
        rows.append(np.stack([np.full_like(i, db), do + i, np.full_like(i, sb), so + i], axis=1))
    if not rows:
        return np.zeros((0, 4), np.int64)
    a = np.concatenate(rows)
    return a[np.lexsort((a[:, 1], a[:, 0]))]


def seg_records(segs, which):
    out = []
    for s in segs:
        local = bool(s["flags"] & ew.EW_SEG_LOCAL)
        data = (64 + int(s["src_owner"])) if s["flags"] & ew.EW_SEG_SNAPSHOT else int(s["holder"])
        if which == 0:
            if not local:
                out.append((data, int(s["src_off"]), 64, int(s["stage_off"]), int(s["len"])))
        elif local or which == 2:   # direct: every segment straight from its source
            out.append((data, int(s["src_off"]), int(s["dst_rank"]), int(s["dst_off"]), int(s["len"])))
        else:
            out.append((128, int(s["stage_off"]), int(s["dst_rank"]), int(s["dst_off"]), int(s["len"])))
    return out


def check_tiles(p, tile_elems, align=0):
    segs = p.segs()
    for which in (0, 1, 2):
        t = p.tiles(which, tile_elems, align)
        assert (t["len"] > 0).all() and (t["len"] <= tile_elems).all()
        got = expand([(int(x["src_buf"]), int(x["src_off"]), int(x["dst_buf"]), int(x["dst_off"]), int(x["len"]))
                      for x in t])
        want = expand(seg_records(segs, which))
        assert got.shape == want.shape and (got == want).all()
        if len(got):  # every destination element written exactly once
            assert (np.diff(got[:, 0] * (1 << 40) + got[:, 1]) > 0).all()


def test_tiles_cover_segments_exactly():
    for (Do, Dn, mask, N, C) in [(4, 3, 0b1011, 8192, 512), (8, 7, 0xFF & ~(1 << 5), 30000 + 8 * 37, 2624),
                                 (7, 8, 0x7F, 20000, 656), (6, 4, 0b111011, 9999, 107), (3, 3, 0b101, 5000, 500),
                                 (5, 9, 0b10101, 8000, 8000), (2, 5, 0b01, 777, 8), (1, 1, 1, 100, 7), (4, 4, 0xF, 0, 8)]:
        p = ew.ew_plan(Do, Dn, mask, N, C)
        for te in (1, 7, 64, 100, 1024, 1 << 20):
            check_tiles(p, te)
        for te, al in ((64, 8), (64, 32), (1024, 32), (2048, 64), (256, 256), (100, 32)):
            check_tiles(p, te, al)
    # explicit boundaries with many different unit lengths: many runs, some of them repeated
    rng = np.random.default_rng(3)
    lens = rng.choice([0, 8, 24, 100, 100, 100, 264, 264, 1000], size=60)
    starts = np.concatenate([[0], np.cumsum(lens)]).astype(np.uint64)
    p = ew.ew_plan_bounds(5, 3, 0b11011, starts)
    assert 1 < p.num_runs <= 60
    for te in (16, 100, 4096):
        check_tiles(p, te)
        check_tiles(p, te, 16)
    assert p.num_tiles(0, 4) == len(p.tiles(0, 1024, 32)) and p.num_tiles(1, 2) == len(p.tiles(1, 2048, 64))


def test_aligned_cuts_fall_on_destination_lines():
    """With the default 128-byte alignment every cut inside a segment is on a 128-byte multiple of
    the destination, and tiles of one destination follow each other front to back."""
    w = configs.stage_7b()
    p = ew.ew_plan(w.old_dp, w.new_dp, w.alive_mask, 40 * w.chunk + 65536, w.chunk)
    segs = p.segs()
    for es, te, al in ((4, 1024, 32), (2, 2048, 64)):
        for which in (0, 1):
            t = p.tiles(which, te, al)
            check = expand([(int(x["src_buf"]), int(x["src_off"]), int(x["dst_buf"]), int(x["dst_off"]), int(x["len"]))
                            for x in t])
            want = expand(seg_records(segs, which))
            assert (check == want).all()
            # segment starts in destination space
            starts = {(int(r[2]), int(r[3])) for r in seg_records(segs, which)}
            for x in t:
                if (int(x["dst_buf"]), int(x["dst_off"])) not in starts:
                    assert int(x["dst_off"]) % al == 0
            # destination-major, ascending inside a destination
            key = t["dst_buf"].astype(np.int64) * (1 << 44) + t["dst_off"].astype(np.int64)
            assert (np.diff(key) > 0).all()
            # few partial tiles: at most two per segment
            assert len(t) <= int(np.ceil(sum(r[4] for r in seg_records(segs, which)) / te)) + 2 * len(segs)


def test_uniform_chunk_plans_are_two_runs():
    w = configs.stage_7b()
    p = ew.ew_plan(w.old_dp, w.new_dp, w.alive_mask, w.numel, w.chunk)
    q = ew.ew_plan_bounds(w.old_dp, w.new_dp, w.alive_mask, w.unit_starts())
    assert p.num_runs == q.num_runs == 2
    assert p.segs().tobytes() == q.segs().tobytes()
    # sampled tiles of the full-size table land inside the buffers they name
    for which, es in ((0, 4), (1, 4), (1, 2)):
        te = 4096 // es
        total = p.num_tiles(which, es)
        for first in (0, total // 2, total - 5):
            out = p.tiles(which, te, 128 // es, first, 5)
            for x in out:
                sb, db = int(x["src_buf"]), int(x["dst_buf"])
                src_cap = p.stage_len if sb == 128 else p.old_shard_len(sb % 64)
                dst_cap = p.stage_len if db == 64 else p.new_shard_len(db)
                assert int(x["src_off"]) + int(x["len"]) <= src_cap
                assert int(x["dst_off"]) + int(x["len"]) <= dst_cap


# ------------------------------------------------------------------ layer migration plans (Sec. 6.3)
def apply_segs(p, old_shards, snaps=None):
    """What pack + unpack must produce, replayed on the host from the explicit segment table."""
    segs = p.segs()
    dt = old_shards[0].dtype
    stage = np.zeros(p.stage_len, dt)
    new = [np.zeros(p.new_shard_len(k), dt) for k in range(p.new_dp)]
    wrote = [np.zeros(p.new_shard_len(k), np.int8) for k in range(p.new_dp)]
    for s in segs:
        src = snaps[int(s["src_owner"])] if s["flags"] & ew.EW_SEG_SNAPSHOT else old_shards[int(s["holder"])]
        a, n = int(s["src_off"]), int(s["len"])
        data = src[a:a + n]
        if not s["flags"] & ew.EW_SEG_LOCAL:
            stage[int(s["stage_off"]):int(s["stage_off"]) + n] = data
            data = stage[int(s["stage_off"]):int(s["stage_off"]) + n]
        k, d = int(s["dst_rank"]), int(s["dst_off"])
        new[k][d:d + n] = data
        wrote[k][d:d + n] += 1
    assert all((w == 1).all() for w in wrote)
    return new


@pytest.mark.parametrize("assignment", [ew.EW_ASSIGN_INTERLEAVED, ew.EW_ASSIGN_CONTIGUOUS])
def test_migrate_plan_equals_oracle(assignment):
    from oracle import migrate
    rng = np.random.default_rng(assignment)
    cases = [(3, [0, 100, 364, 1000], [0, 264, 500], 2), (4, [0, 8, 16, 4099], [0, 7], 1), (2, [0, 50, 120], [0, 30, 90, 91], 0),
             (5, [0, 1000], [0, 24, 48], 1), (4, list(range(0, 4097, 256)), list(range(0, 2049, 256)), 5),
             (8, list(range(0, 64 * 641, 640)), list(range(0, 64 * 321, 640)), 7), (1, [0, 9, 30], [0, 5], 2),
             (32, [0, 5000, 10000], [0, 5000], 1)]
    for D, src, dst, n_move in cases:
        src, dst = np.asarray(src, np.int64), np.asarray(dst, np.int64)
        s_iv = migrate.rank_intervals(src, D, assignment)
        d_iv = migrate.rank_intervals(dst, D, assignment)
        s_sh = [rng.integers(0, 1 << 40, sum(h - l for l, h in x)) for x in s_iv]
        d_sh = [rng.integers(0, 1 << 40, sum(h - l for l, h in x)) for x in d_iv]
        want_s, want_d = migrate.migrate(s_sh, d_sh, src, dst, D, assignment, n_move)
        p = ew.ew_plan_migrate(assignment, D, src, dst, n_move)
        assert p.old_dp == p.new_dp == 2 * D
        assert [p.old_shard_len(r) for r in range(2 * D)] == [len(x) for x in s_sh + d_sh]
        assert [p.new_shard_len(r) for r in range(2 * D)] == [len(x) for x in want_s + want_d]
        got = apply_segs(p, s_sh + d_sh)
        for a, b in zip(got, want_s + want_d):
            assert np.array_equal(a, b)
        # traffic matrix = the oracle's ownership-change matrix
        m = migrate.traffic(src, dst, D, assignment, n_move)
        segs = p.segs()
        for h in range(2 * D):
            for k in range(2 * D):
                if h != k:
                    assert p.pair_len(h, k) == m[h, k]
                else:
                    sel = segs[(segs["holder"] == h) & (segs["dst_rank"] == k)]
                    assert int(sel["len"].sum()) == m[h, k]
        check_invariants(p, 2 * D, 2 * D, (1 << (2 * D)) - 1, int(src[-1] + dst[-1]))
        for te, al in ((64, 0), (1024, 32)):
            check_tiles(p, te, al)


def test_migrate_closed_forms_at_the_paper_degree():
    # Llama2-34B workload of the paper: DP 3 (Table 2); one layer of the 7B shape stands in for |O_i|
    layer = sum(configs.llama_layer_tensors(4096, 11008))
    D = 3
    units = 24
    L = layer // units              # 8 432 640: a multiple of 8 * D
    assert L * units == layer and L % (8 * D * D) == 0
    src = np.arange(4 * units + 1, dtype=np.uint64) * L   # 4 layers on stage S
    dst = np.arange(4 * units + 1, dtype=np.uint64) * L   # 4 layers on stage S+1
    pi = ew.ew_plan_migrate(ew.EW_ASSIGN_INTERLEAVED, D, src, dst, units)
    pc = ew.ew_plan_migrate(ew.EW_ASSIGN_CONTIGUOUS, D, src, dst, units)
    pairs = {(h, k): pi.pair_len(h, k) for h in range(2 * D) for k in range(2 * D) if pi.pair_len(h, k)}
    assert pairs == {(j, D + j): layer // D for j in range(D)}        # exactly D 1:1 sends summing to |O_i|
    assert pi.stage_len == layer
    cross = sum(pc.pair_len(h, k) for h in range(D) for k in range(D, 2 * D))
    intra_s = sum(pc.pair_len(h, k) for h in range(D) for k in range(D))
    intra_d = sum(pc.pair_len(h, k) for h in range(D, 2 * D) for k in range(D, 2 * D))
    assert cross == layer and 2 * intra_s == (D - 1) * layer and 2 * intra_d == (D - 1) * layer
    assert 2 * (cross + intra_s) == (D + 1) * layer                    # the paper's (D+1)/2 |O_i|
    assert pi.num_runs == 3 and pc.num_runs == 1


def test_migrate_errors():
    def code(*a):
        with pytest.raises(ew.EwError) as e:
            ew.ew_plan_migrate(*a)
        return e.value.code
    assert code(2, 4, [0, 8], [0, 8], 1) == ew.EW_EINVAL          # unknown assignment
    assert code(0, 0, [0, 8], [0, 8], 1) == ew.EW_EINVAL
    assert code(0, 33, [0, 8], [0, 8], 1) == ew.EW_EINVAL         # 2*dp > 64
    assert code(0, 4, [0, 8], [0, 8], 2) == ew.EW_EINVAL          # more layers than the stage has
    assert code(1, 4, [0, 8, 4], [0, 8], 1) == ew.EW_EINVAL


def test_header_is_plain_c(tmp_path, repo_root):
    """The boundary is a C ABI: the header must compile as C99 on its own, and a C program must link
    against the library and plan a reshard (host-only calls)."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if not gcc:
        pytest.skip("no C compiler")
    src = tmp_path / "use.c"
    src.write_text(r'''
#include "elaswave.h"
#include <stdio.h>
int main(void) {
  ew_plan_t *p = 0;
  int rc = ew_plan(4, 3, 0xB, 1u << 20, 4096, &p);
  if (rc != EW_OK) { printf("plan failed: %s\n", ew_strerror(rc)); return 1; }
  printf("%llu %llu %d\n", (unsigned long long)ew_plan_num_segs(p), (unsigned long long)ew_plan_stage_len(p),
         (int)ew_plan_new_rank_of(p, 3));
  ew_plan_free(p);
  return sizeof(ew_seg_t) == 40 && sizeof(ew_cksum_t) == 16 && sizeof(ew_adam_t) == 36 ? 0 : 2;
}
''')
    exe = tmp_path / "use"
    libdir = os.path.dirname(binding.LIB_PATH)
    subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(repo_root, "include"), str(src),
                    "-o", str(exe), "-L", libdir, "-l:libelaswave.so", f"-Wl,-rpath,{libdir}"], check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.split() == ["1536", "174080", "2"]


# ------------------------------------------------------------------ randomised: any boundaries, any membership
def test_random_boundaries_and_memberships_match_the_oracle():
    from hypothesis import given, settings, strategies as st

    @st.composite
    def cases(draw):
        old_dp = draw(st.integers(1, 9))
        new_dp = draw(st.integers(1, 9))
        alive = [draw(st.booleans()) for _ in range(old_dp)]
        for j in range(old_dp):          # make it recoverable: a failed rank's predecessor survives
            if not alive[j] and not alive[(j - 1) % old_dp]:
                alive[(j - 1) % old_dp] = True
        if not any(alive):
            alive[0] = True
        for j in range(old_dp):
            if not alive[j] and not alive[(j - 1) % old_dp]:
                alive[j] = True
        lens = draw(st.lists(st.sampled_from([0, 1, 7, 8, 16, 24, 100, 264, 1000]), min_size=0, max_size=12))
        return old_dp, new_dp, sum(1 << j for j, a in enumerate(alive) if a), lens

    @settings(max_examples=150, deadline=None, derandomize=True, database=None)
    @given(cases())
    def run(case):
        old_dp, new_dp, mask, lens = case
        starts = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        alive = layout.alive_list(old_dp, mask)
        layout.check_recoverable(old_dp, alive)
        rng = np.random.default_rng(int(starts[-1]) + old_dp * 100 + new_dp)
        olen = layout.shard_lengths(starts, old_dp)
        data = [rng.integers(0, 1 << 40, n) for n in olen]
        want = layout.reshard([d if alive[j] else None for j, d in enumerate(data)],
                              [None if alive[j] else d for j, d in enumerate(data)], old_dp, new_dp, mask, starts)
        p = ew.ew_plan_bounds(old_dp, new_dp, mask, starts.astype(np.uint64))
        poison = [d if alive[j] else np.full_like(d, -1) for j, d in enumerate(data)]
        got = apply_segs(p, poison, data)
        assert len(got) == len(want)
        for a, b in zip(got, want):
            assert np.array_equal(a, b)
        check_tiles(p, 64, 16)

    run()


def test_xcd_remap_is_a_permutation_of_every_launch():
    """The workgroup -> tile mapping of the tile kernels, checked through the library's own decoder on
    the host: for every launch size and group size the mapped ids are a permutation of 0..n-1, runs of
    `group` consecutive tiles land on one residue class mod 8 (one XCD), and a trailing partial block
    keeps the identity."""
    fn = ew.ew_tile_of_workgroup
    for n in (0, 1, 7, 8, 9, 63, 64, 65, 511, 512, 513, 1000, 4097):
        for g in (0, 1, 2, 3, 8, 64, 512, 5000):
            got = [fn(w, n, g) for w in range(n)]
            assert sorted(got) == list(range(n)), (n, g)
            if g > 1:
                blk = 8 * g
                for w in range(n):
                    base = w // blk * blk
                    if base + blk <= n:      # full block: XCD w % 8 owns tiles base + (w%8)*g .. +g-1
                        assert (got[w] - base) // g == w % 8
                    else:
                        assert got[w] == w
