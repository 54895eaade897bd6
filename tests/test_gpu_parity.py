"""GPU parity tests: the HIP path (through the C ABI) against the CPU oracle, bit for bit.
Small and ragged cases here; the five named workloads are in test_gpu_workloads.py."""
import numpy as np
import pytest
import torch

import paper_2510_00606_amd as ew
from oracle import checksum, layout

from gpu_util import DEV, GUARD, guard_intact, guarded, np_bits, random_shards, run_reshard, stream, to_dev

pytestmark = pytest.mark.gpu

MIB = 1 << 20


@pytest.fixture(autouse=True)
def default_params():
    saved = {k: ew.ew_get_param(k) for k in ("tile_bytes", "tile_elems", "tile_align_bytes", "cksum_sub_bytes", "cksum_wgs_per_cu",
                                              "cksum_mode", "fused_wgs_per_cu", "fused_mode", "verify_wgs_per_cu",
                                              "snapshot_wave_min_bytes", "xcd_group_kib", "snapshot_xcd_group_kib",
                                              "fold_tiles_per_lane", "fused_pass_tiles", "verify_large_min_bytes", "verify_large_sub_bytes",
                                              "verify_large_wgs_per_cu")}
    yield
    for k, v in saved.items():
        ew.ew_set_param(k, v)


# ------------------------------------------------------------------ snapshot + checksum
def snapshot_case(nbytes, rng, src_shift=0, dst_shift=0):
    raw = rng.integers(0, 256, nbytes + 64, dtype=np.uint8)
    src_all = torch.from_numpy(raw).to(DEV)
    src = src_all[src_shift:src_shift + nbytes]
    dst_all = torch.full((nbytes + 128,), 0x5A, dtype=torch.uint8, device=DEV)
    dst = dst_all[dst_shift:dst_shift + nbytes]
    nb = ew.num_blocks(nbytes)
    ck = torch.full((nb + 1, 2), -1, dtype=torch.int64, device=DEV)
    ew.ew_snapshot(src, dst, nbytes, ck, stream())
    torch.cuda.synchronize()
    host = raw[src_shift:src_shift + nbytes]
    assert np.array_equal(dst.cpu().numpy(), host), "snapshot bytes differ"
    assert bool((dst_all[:dst_shift] == 0x5A).all()) and bool((dst_all[dst_shift + nbytes:] == 0x5A).all())
    want = checksum.block_checksums(host)
    got = ck.cpu().numpy().view(np.uint64)
    assert np.array_equal(got[:nb], want), "checksums differ"
    assert (got[nb] == np.uint64((1 << 64) - 1)).all(), "record past the end was written"


SIZES = [0, 1, 7, 8, 9, 15, 16, 17, 255, 4096, 4096 * 3 + 5, 65536, 65536 + 16, 65536 * 5 - 3, MIB - 16, MIB - 1, MIB,
         MIB + 1, MIB + 8, MIB + 4096, 3 * MIB + 12345, 17 * MIB + 65536 + 24]


@pytest.mark.parametrize("nbytes", SIZES)
def test_snapshot_matches_oracle(nbytes):
    snapshot_case(nbytes, np.random.default_rng(nbytes))


@pytest.mark.parametrize("nbytes", SIZES)
def test_snapshot_one_wave_shape_on_small_buffers(nbytes):
    """The shape meant for large buffers, forced on every size."""
    ew.ew_set_param("snapshot_wave_min_bytes", 0)
    snapshot_case(nbytes, np.random.default_rng(nbytes + 1))


@pytest.mark.parametrize("kib", [0, 4, 12, 128, 1 << 20])
@pytest.mark.parametrize("wave_min", [0, 1 << 62])
def test_snapshot_chunks_dealt_to_xcds_in_runs(kib, wave_min):
    """Runs of chunks per XCD permute which workgroup takes which chunk (and which slot it writes),
    never the result: both workgroup shapes, run lengths that do not divide the launch, runs longer
    than the launch."""
    ew.ew_set_param("snapshot_xcd_group_kib", kib)
    ew.ew_set_param("snapshot_wave_min_bytes", wave_min)
    for nbytes in (1, 4097, MIB - 8, 3 * MIB + 12345, 17 * MIB + 65536 + 24):
        snapshot_case(nbytes, np.random.default_rng(kib + nbytes))


@pytest.mark.parametrize("sub,wgs", [(4096, 0), (16384, 2), (65536, 0), (262144, 1), (MIB, 0), (MIB, 3)])
def test_snapshot_launch_shapes(sub, wgs):
    ew.ew_set_param("cksum_mode", 1)   # the scratch-free atomic kernel
    ew.ew_set_param("cksum_sub_bytes", sub)
    ew.ew_set_param("cksum_wgs_per_cu", wgs)
    for nbytes in (1, 4097, MIB - 8, 9 * MIB + 100000 + 3, 64 * MIB):
        snapshot_case(nbytes, np.random.default_rng(sub + wgs + nbytes))


@pytest.mark.parametrize("shift", [(1, 0), (0, 3), (8, 8), (5, 11)])
def test_snapshot_unaligned_buffers(shift):
    for nbytes in (1, 100, 4096 + 7, 2 * MIB + 77):
        snapshot_case(nbytes, np.random.default_rng(nbytes + shift[0]), *shift)


def test_snapshot_closed_forms():
    n = 131072  # words in one block
    for words, want in ((np.zeros(n, np.uint64), (0, 0)),
                        (np.full(n, (1 << 64) - 1, np.uint64), ((-n) % (1 << 64), 0)),
                        (np.arange(n, dtype=np.uint64), (8589869056, 0))):
        src = torch.from_numpy(words.view(np.int64)).to(DEV)
        dst = torch.empty_like(src)
        ck = torch.zeros((1, 2), dtype=torch.int64, device=DEV)
        ew.ew_snapshot(src, dst, n * 8, ck, stream())
        got = ck.cpu().numpy().view(np.uint64)[0]
        assert (int(got[0]), int(got[1])) == want


# ------------------------------------------------------------------ verify
def verify_case(nbytes, flips, rng, cap=16):
    raw = rng.integers(0, 256, nbytes, dtype=np.uint8)
    buf = torch.from_numpy(raw).to(DEV)
    nb = ew.num_blocks(nbytes)
    snap = torch.empty_like(buf)
    stored = torch.zeros((max(nb, 1), 2), dtype=torch.int64, device=DEV)
    ew.ew_snapshot(buf, snap, nbytes, stored, stream())
    torch.cuda.synchronize()
    host = raw.copy()
    for (o, bit) in flips:
        host[o] ^= np.uint8(1 << bit)
        snap[o] ^= (1 << bit)
    got = torch.full((max(nb, 1), 2), -1, dtype=torch.int64, device=DEV)
    n_bad = torch.full((1,), -1, dtype=torch.int64, device=DEV)
    bad = torch.full((cap + 1,), -1, dtype=torch.int64, device=DEV)
    diffs = torch.full((cap + 1, 2), -1, dtype=torch.int64, device=DEV)
    ew.ew_verify(snap, nbytes, stored, got, n_bad, bad, diffs, cap, stream())
    torch.cuda.synchronize()
    o_bad, o_diffs = checksum.verify(host, stored.cpu().numpy().view(np.uint64)[:nb])
    assert np.array_equal(stored.cpu().numpy().view(np.uint64)[:nb], checksum.block_checksums(raw))
    assert int(n_bad.item()) == len(o_bad)
    m = min(len(o_bad), cap)
    assert bad.cpu().numpy()[:m].tolist() == o_bad[:m].tolist()
    assert np.array_equal(diffs.cpu().numpy().view(np.uint64)[:m], o_diffs[:m])
    assert bad.cpu().numpy()[m:].tolist() == [-1] * (cap + 1 - m), "bad-block list written past the count/cap"
    if nb:
        assert np.array_equal(got.cpu().numpy().view(np.uint64)[:nb], checksum.block_checksums(host))
    return o_bad, o_diffs


@pytest.mark.parametrize("mode", [-1, 0, 1])
def test_verify_clean_and_single_flip(mode):
    ew.ew_set_param("cksum_mode", mode)
    rng = np.random.default_rng(42)
    nbytes = 21 * MIB + 4096 + 5
    bad, _ = verify_case(nbytes, [], rng)
    assert len(bad) == 0
    for _ in range(4):
        o, bit = int(rng.integers(0, nbytes)), int(rng.integers(0, 8))
        bad, diffs = verify_case(nbytes, [(o, bit)], rng)
        assert bad.tolist() == [o >> 20]
        assert int(diffs[0, 1]) == 1 << (8 * (o % 8) + bit)


@pytest.mark.parametrize("wgs", [0, 1, 2, 4, 8])
def test_verify_with_occupancy_caps(wgs):
    """The cap on resident workgroups changes the launch only, never the result."""
    ew.ew_set_param("verify_wgs_per_cu", wgs)
    rng = np.random.default_rng(90 + wgs)
    nbytes = 9 * MIB + 4096 * 3 + 11
    o, bit = int(rng.integers(0, nbytes)), int(rng.integers(0, 8))
    bad, diffs = verify_case(nbytes, [(o, bit)], rng)
    assert bad.tolist() == [o >> 20] and int(diffs[0, 1]) == 1 << (8 * (o % 8) + bit)


@pytest.mark.parametrize("sub,wgs", [(262144, 2), (4096, 0), (1 << 20, 1), (65536, 8)])
def test_verify_with_the_launch_shape_for_large_buffers(sub, wgs):
    """The shape that large read-only passes take (fewer, longer streams), forced on small and ragged
    buffers: it changes the launch only, never the result."""
    ew.ew_set_param("verify_large_min_bytes", 0)
    ew.ew_set_param("verify_large_sub_bytes", sub)
    ew.ew_set_param("verify_large_wgs_per_cu", wgs)
    rng = np.random.default_rng(120 + wgs)
    for nbytes in (1, 4097, MIB - 8, 9 * MIB + 100000 + 3, 40 * MIB + 24):
        o, bit = int(rng.integers(0, nbytes)), int(rng.integers(0, 8))
        bad, diffs = verify_case(nbytes, [(o, bit)], rng)
        assert bad.tolist() == [o >> 20] and int(diffs[0, 1]) == 1 << (8 * (o % 8) + bit)


def test_verify_many_flips_ordered_and_capped():
    rng = np.random.default_rng(43)
    nbytes = 2100 * MIB // 100  # 21 MiB
    flips = [(b * MIB + int(rng.integers(0, MIB)), int(rng.integers(0, 8))) for b in (20, 3, 11, 0, 7, 15)]
    bad, _ = verify_case(nbytes, flips, rng)
    assert bad.tolist() == [0, 3, 7, 11, 15, 20]
    verify_case(nbytes, flips, rng, cap=4)
    verify_case(nbytes, flips, rng, cap=0)
    verify_case(0, [], rng)
    # more blocks than one compare pass (1024 threads) with flips in several passes
    nbytes = 2500 * MIB
    big = [(b * MIB + 17, 1) for b in (5, 1023, 1024, 2047, 2048, 2499)]
    bad, _ = verify_case(nbytes, big, rng)
    assert bad.tolist() == [5, 1023, 1024, 2047, 2048, 2499]


# ------------------------------------------------------------------ pack / unpack
def reshard_case(old_dp, new_dp, mask, numel, chunk, elem_size, rng, tile_elems=0, starts=None):
    """Uniform chunk, or explicit unit boundaries `starts` (then numel and chunk are ignored)."""
    explicit = starts is not None
    if explicit:
        starts = np.asarray(starts, dtype=np.int64)
        numel = int(starts[-1])
    else:
        starts = layout.unit_starts(numel, chunk)
    alive = layout.alive_list(old_dp, mask)
    lens = layout.shard_lengths(starts, old_dp)
    data = random_shards(lens, elem_size, rng)   # the true content of every old rank's partition
    poison = 0xDEAD if elem_size == 2 else 0xDEADBEEF
    o_shards = [d if alive[j] else None for j, d in enumerate(data)]
    o_snaps = [None if alive[j] else d for j, d in enumerate(data)]
    want_new = layout.reshard(o_shards, o_snaps, old_dp, new_dp, mask, starts)
    want_stage, want_table = layout.staging(o_shards, o_snaps, old_dp, new_dp, mask, starts)

    # device: failed ranks' live shards are poisoned, alive ranks have no snapshot at all
    old_dev = [to_dev(d if alive[j] else np.full_like(d, poison), elem_size) for j, d in enumerate(data)]
    snap_dev = [None if alive[j] else to_dev(d, elem_size) for j, d in enumerate(data)]
    plan = ew.ew_plan_bounds(old_dp, new_dp, mask, starts) if explicit else ew.ew_plan(old_dp, new_dp, mask, numel, chunk)
    stage, new = run_reshard(plan, old_dev, snap_dev, elem_size, tile_elems)

    assert plan.stage_len == len(want_stage)
    assert np.array_equal(np_bits(stage[:plan.stage_len]), want_stage), "staging arena differs"
    assert guard_intact(stage, plan.stage_len, elem_size)
    for (h, k), (off, n) in want_table.items():
        assert (plan.pair_off(h, k), plan.pair_len(h, k)) == (off, n)
    for k in range(new_dp):
        n = plan.new_shard_len(k)
        assert n == len(want_new[k])
        assert np.array_equal(np_bits(new[k][:n]), want_new[k]), f"new shard {k} differs"
        assert guard_intact(new[k], n, elem_size)

    # direct form: every segment pulled straight from its source, no arena
    new_d = [guarded(plan.new_shard_len(k), elem_size) for k in range(new_dp)]
    ew.ew_reshard(plan, old_dev, snap_dev, new_d, elem_size, stream())
    torch.cuda.synchronize()
    for k in range(new_dp):
        n = plan.new_shard_len(k)
        assert np.array_equal(np_bits(new_d[k][:n]), want_new[k]), f"direct: new shard {k} differs"
        assert guard_intact(new_d[k], n, elem_size)

    # fused form: unpack + snapshot + checksums of the new shards in one pass
    new2 = [guarded(plan.new_shard_len(k), elem_size) for k in range(new_dp)]
    snap2 = [guarded(plan.new_shard_len(k), elem_size) for k in range(new_dp)]
    nblk = [ew.num_blocks(plan.new_shard_len(k) * elem_size) for k in range(new_dp)]
    ck2 = [torch.full((nb + 1, 2), -1, dtype=torch.int64, device=DEV) for nb in nblk]
    if tile_elems * elem_size > MIB and numel > 0:   # a tile may span at most two checksum blocks
        with pytest.raises(ew.EwError) as e:
            ew.ew_unpack_snapshot(plan, stage, old_dev, snap_dev, new2, snap2, ck2, elem_size, stream())
        assert e.value.code == ew.EW_EINVAL
        plan.close()
        return
    ew.ew_unpack_snapshot(plan, stage, old_dev, snap_dev, new2, snap2, ck2, elem_size, stream())
    torch.cuda.synchronize()
    for k in range(new_dp):
        n = plan.new_shard_len(k)
        assert np.array_equal(np_bits(new2[k][:n]), want_new[k]), f"fused: new shard {k} differs"
        assert np.array_equal(np_bits(snap2[k][:n]), want_new[k]), f"fused: snapshot of new shard {k} differs"
        assert guard_intact(new2[k], n, elem_size) and guard_intact(snap2[k], n, elem_size)
        got = ck2[k].cpu().numpy().view(np.uint64)
        assert np.array_equal(got[:nblk[k]], checksum.block_checksums(want_new[k])), f"fused: checksums of {k} differ"
        assert (got[nblk[k]] == np.uint64((1 << 64) - 1)).all(), "record past the end was written"
    # ... and the same without the arena
    new3 = [guarded(plan.new_shard_len(k), elem_size) for k in range(new_dp)]
    snap3 = [guarded(plan.new_shard_len(k), elem_size) for k in range(new_dp)]
    ck3 = [torch.full((nb + 1, 2), -1, dtype=torch.int64, device=DEV) for nb in nblk]
    ew.ew_reshard_snapshot(plan, old_dev, snap_dev, new3, snap3, ck3, elem_size, stream())
    torch.cuda.synchronize()
    for k in range(new_dp):
        n = plan.new_shard_len(k)
        assert np.array_equal(np_bits(new3[k][:n]), want_new[k]), f"direct fused: new shard {k} differs"
        assert np.array_equal(np_bits(snap3[k][:n]), want_new[k]), f"direct fused: snapshot of new shard {k} differs"
        assert guard_intact(new3[k], n, elem_size) and guard_intact(snap3[k], n, elem_size)
        assert torch.equal(ck3[k], ck2[k]), f"direct fused: checksums of {k} differ"
    plan.close()


def recoverable_masks(old_dp):
    return [m for m in range(1, 1 << old_dp)
            if all((m >> j) & 1 or (m >> ((j - 1) % old_dp)) & 1 for j in range(old_dp))]


@pytest.mark.parametrize("elem_size", [2, 4])
def test_reshard_small_exhaustive(elem_size):
    rng = np.random.default_rng(elem_size)
    for Do in range(1, 5):
        for Dn in range(1, 5):
            for mask in recoverable_masks(Do):
                for N, C in ((0, 8), (1, 1), (9, 8), (64, 24), (1000, 24), (1000, 100), (4099, 264), (4099, 5000)):
                    reshard_case(Do, Dn, mask, N, C, elem_size, rng)


@pytest.mark.parametrize("elem_size", [2, 4])
@pytest.mark.parametrize("case", [
    (4, 3, 0b1011, 1 << 20, 4096),            # the paper's scenario at the Tiny workload's size
    (8, 7, 0xFF & ~(1 << 5), 3_000_000 + 8 * 37, 262144),   # several tiles per segment, ragged tail unit
    (7, 8, 0x7F, 2_000_000, 65536),           # scale-up with a joiner
    (16, 12, 0xFFFF & ~0b0101001000000010, 1_500_000 + 104, 4096),  # 4 failures
    (6, 4, 0b111111, 999_999, 10_007),        # voluntary shrink, nothing aligned
    (3, 3, 0b101, 500_000, 50_000),           # same degree, one rank replaced from its snapshot
    (5, 9, 0b10101, 800_000, 800_000),        # one unit, two failures, growth
    (3, 2, 0b111, 2_600_000, 99_992),         # new shards of several checksum blocks, tiles straddling them
    (2, 3, 0b10, 1_900_003, 70_001),          # ragged units: words split between segments
    (64, 63, (1 << 63) - 1, 64 * 63 * 8 * 3 + 40, 64 * 63 * 8),   # the largest degree, last rank failed
    (64, 32, 0x5555555555555555, 1_000_000, 40_000),               # every second rank failed: 32 snapshots in use
    (1, 64, 0b1, 300_000, 30_000),            # scatter from one rank to the largest degree
    (64, 1, (1 << 64) - 1, 300_000, 30_000),  # gather from the largest degree
])
def test_reshard_medium(case, elem_size):
    rng = np.random.default_rng(hash(case) & 0xFFFF)
    reshard_case(*case, elem_size, rng)


@pytest.mark.parametrize("tile_elems,align", [(0, 128), (0, 0), (0, 64), (64, 128), (1000, 16), (4096, 256), (8192, 0), (65536, 128),
                                              (1 << 20, 128)])
def test_reshard_launch_shapes(tile_elems, align):
    ew.ew_set_param("tile_align_bytes", align)
    rng = np.random.default_rng(tile_elems)
    for es in (2, 4):
        reshard_case(8, 7, 0xFF & ~(1 << 5), 3_000_000 + 8 * 37, 262144, es, rng, tile_elems)
        reshard_case(6, 4, 0b111011, 999_999, 10_007, es, rng, tile_elems)


def random_unit_lengths(rng):
    """A mix of what real boundary lists contain: runs of equal units, tensors of odd sizes, empty
    and tiny units, lengths that are not multiples of the 8-element granule."""
    lens = []
    for _ in range(int(rng.integers(1, 9))):
        kind = int(rng.integers(0, 6))
        if kind == 0:
            lens += [int(rng.integers(1, 40)) * 8 * int(rng.integers(1, 200))] * int(rng.integers(2, 12))   # a run
        elif kind == 1:
            lens.append(int(rng.integers(0, 60)))                       # tiny or empty
        elif kind == 2:
            lens.append(int(rng.integers(1, 30_000)))                   # ragged
        elif kind == 3:
            lens.append(8 * int(rng.integers(1, 40_000)))               # granule multiple, several tiles
        elif kind == 4:
            lens += [int(rng.integers(1, 2_000))] * int(rng.integers(2, 6))   # a run of ragged units
        else:
            lens.append(1024 * int(rng.integers(1, 300)))               # tile multiple
    return lens


@pytest.mark.parametrize("seed", range(48))
def test_reshard_random_unit_boundaries(seed):
    rng = np.random.default_rng(1000 + seed)
    old_dp, new_dp = int(rng.integers(1, 10)), int(rng.integers(1, 10))
    masks = recoverable_masks(old_dp)
    mask = masks[int(rng.integers(0, len(masks)))]
    starts = np.concatenate([[0], np.cumsum(random_unit_lengths(rng))])
    ew.ew_set_param("tile_align_bytes", int(rng.choice([0, 16, 128, 256])))
    tile_elems = int(rng.choice([0, 0, 256, 1024, 3000]))
    reshard_case(old_dp, new_dp, mask, None, None, 2 + 2 * (seed & 1), rng, tile_elems, starts=starts)


@pytest.mark.parametrize("wgs", [0, 2, 3, 5, 7, 8])
def test_fused_unpack_with_occupancy_caps(wgs):
    """The cap on resident workgroups changes the launch (dynamic LDS), never the result."""
    ew.ew_set_param("fused_wgs_per_cu", wgs)
    rng = np.random.default_rng(200 + wgs)
    for es in (2, 4):
        reshard_case(8, 7, 0xFF & ~(1 << 5), 3_000_000 + 8 * 37, 262144, es, rng)
        reshard_case(3, 2, 0b111, 2_600_000, 99_992, es, rng)


@pytest.mark.parametrize("kib", [0, 4, 8, 12, 64, 2048, 1 << 20])
def test_tiles_dealt_to_xcds_in_runs(kib):
    """The workgroup -> tile mapping (runs of consecutive tiles per XCD) permutes who copies which tile,
    never what is copied: every group size, also ones that do not divide the number of tiles, tiles
    that are smaller than nominal, and groups larger than the launch."""
    ew.ew_set_param("xcd_group_kib", kib)
    rng = np.random.default_rng(500 + kib)
    for es in (2, 4):
        reshard_case(8, 7, 0xFF & ~(1 << 5), 3_000_000 + 8 * 37, 262144, es, rng)
        reshard_case(3, 2, 0b111, 2_600_000, 99_992, es, rng)
        reshard_case(6, 4, 0b111011, 999_999, 10_007, es, rng, tile_elems=1000)
        reshard_case(4, 3, 0b1011, 4099, 264, es, rng)


@pytest.mark.parametrize("per_lane", [1, 3, 16, 1000])
def test_fused_fold_with_any_number_of_tiles_per_lane(per_lane):
    """How many tiles a lane of the fold kernel walks changes how the slots meet in the records, never the
    records: one tile per lane, counts that do not divide a block's tiles, more tiles per lane than a pass has."""
    ew.ew_set_param("fold_tiles_per_lane", per_lane)
    rng = np.random.default_rng(700 + per_lane)
    for es in (2, 4):
        reshard_case(8, 7, 0xFF & ~(1 << 5), 3_000_000 + 8 * 37, 262144, es, rng)
        reshard_case(3, 2, 0b111, 2_600_000, 99_992, es, rng)
        reshard_case(2, 3, 0b10, 1_900_003, 70_001, es, rng)


@pytest.mark.parametrize("per_launch", [0, 1, 7, 100, 4096])
def test_fused_unpack_in_several_launches(per_launch):
    """The fused kernel's tiles go out in launches of a bounded size with one fold at the end: any bound,
    also one that leaves a ragged last launch or exceeds the table, gives the oracle's bits, with and
    without a scratch region."""
    ew.ew_set_param("fused_pass_tiles", per_launch)
    for mode in (0, 1):
        ew.ew_set_param("fused_mode", mode)
        rng = np.random.default_rng(900 + per_launch + mode)
        reshard_case(5, 4, 0b10111, 3 * 4096 * 40 + 8 * 11, 4096, 4, rng)
        reshard_case(4, 6, 0b1111, 250_000 * 8, 50_000 * 8, 2, rng, tile_elems=256)


def test_fused_unpack_scratch_free_form():
    """The form a graph capture falls back to when it can get no scratch region: every workgroup adds
    its tile to the records with atomics.  Same bits as the slot form and as the oracle."""
    ew.ew_set_param("fused_mode", 1)
    rng = np.random.default_rng(321)
    for es in (2, 4):
        reshard_case(8, 7, 0xFF & ~(1 << 5), 3_000_000 + 8 * 37, 262144, es, rng)
        reshard_case(3, 2, 0b111, 2_600_000, 99_992, es, rng)      # tiles straddling checksum blocks
        reshard_case(2, 3, 0b10, 1_900_003, 70_001, es, rng)       # ragged units: words split between segments
        reshard_case(4, 3, 0b1011, 4099, 264, es, rng)


# ------------------------------------------------------------------ a run of failures and joins
@pytest.mark.parametrize("elem_size", [2, 4])
def test_chain_of_failures_and_joins(elem_size):
    """Sec. 5.1 + 5.2 over several events: what the fused unpack leaves behind (new shards, their
    snapshot copies, their checksums) is what the next event recovers from.  After every event the
    new shards are the oracle's slices of the one flat array that never changes, the snapshot copies
    equal them, the checksums are the oracle's, and the snapshot a recovery is about to read
    verifies clean -- once after a planted bit flip was found and undone."""
    rng = np.random.default_rng(700 + elem_size)
    cuts = np.unique(np.concatenate([[0], rng.integers(1, 900_000, 37) * 8, [900_000 * 8 + 8 * 13]]))
    starts = cuts.astype(np.int64)
    npdt = {2: np.uint16, 4: np.uint32}[elem_size]
    flat = rng.integers(0, 1 << (8 * elem_size), size=int(starts[-1]), dtype=np.uint64).astype(npdt)
    dp = 8
    want = layout.slice_flat(flat, dp, starts)
    shards = [to_dev(a, elem_size) for a in want]
    snaps, cks = [], []
    for a, t in zip(want, shards):          # the first snapshots come from ew_snapshot
        sn = torch.empty_like(t)
        ck = torch.zeros((ew.num_blocks(a.nbytes), 2), dtype=torch.int64, device=DEV)
        ew.ew_snapshot(t, sn, a.nbytes, ck, stream())
        snaps.append(sn)
        cks.append(ck)
    events = [(7, [5]), (8, []), (6, [1, 4]), (4, [0, 2]), (5, [3]), (5, [1, 3]), (1, [0, 2]), (3, [])]
    poison = 0xDEAD if elem_size == 2 else 0xDEADBEEF
    for step, (new_dp, failed) in enumerate(events):
        mask = sum(1 << j for j in range(dp) if j not in failed)
        for j in failed:
            shards[j].fill_(poison - (1 << (8 * elem_size)))     # the live shard is gone
            nbytes = want[j].nbytes
            nb = ew.num_blocks(nbytes)
            got = torch.zeros((nb, 2), dtype=torch.int64, device=DEV)
            n_bad = torch.zeros(1, dtype=torch.int64, device=DEV)
            bad = torch.full((4,), -1, dtype=torch.int64, device=DEV)
            diffs = torch.zeros((4, 2), dtype=torch.int64, device=DEV)
            if step == 2 and j == failed[0]:      # a flipped bit in the snapshot is found, then undone
                o, bit = int(rng.integers(0, nbytes)), int(rng.integers(0, 8))
                raw = snaps[j].view(torch.uint8)
                raw[o] ^= (1 << bit)
                ew.ew_verify(snaps[j], nbytes, cks[j], got, n_bad, bad, diffs, 4, stream())
                torch.cuda.synchronize()
                assert int(n_bad.item()) == 1 and int(bad[0].item()) == o >> 20
                d = diffs.cpu().numpy().view(np.uint64)[0]
                lane, direction = ew.ew_single_bit_flip(int(d[0]), int(d[1]))
                assert lane == 8 * (o % 8) + bit
                raw[o] ^= (1 << bit)
            ew.ew_verify(snaps[j], nbytes, cks[j], got, n_bad, bad, diffs, 4, stream())
            torch.cuda.synchronize()
            assert int(n_bad.item()) == 0, f"event {step}: snapshot of rank {j} does not verify"
        plan = ew.ew_plan_bounds(dp, new_dp, mask, starts)
        ew.ew_plan_upload(plan, 0, stream())
        stage = guarded(plan.stage_len, elem_size)
        alive_snaps = [snaps[j] if j in failed else None for j in range(dp)]
        ew.ew_pack(plan, shards, alive_snaps, stage, elem_size, stream())
        lens = [plan.new_shard_len(k) for k in range(new_dp)]
        new = [guarded(n, elem_size) for n in lens]
        new_snaps = [guarded(n, elem_size) for n in lens]
        new_cks = [torch.full((ew.num_blocks(n * elem_size) + 1, 2), -1, dtype=torch.int64, device=DEV) for n in lens]
        ew.ew_unpack_snapshot(plan, stage, shards, alive_snaps, new, new_snaps, new_cks, elem_size, stream())
        torch.cuda.synchronize()
        plan.close()
        want = layout.slice_flat(flat, new_dp, starts)
        for k in range(new_dp):
            n = lens[k]
            assert n == len(want[k])
            assert np.array_equal(np_bits(new[k][:n]), want[k]), f"event {step}: new shard {k} differs"
            assert np.array_equal(np_bits(new_snaps[k][:n]), want[k]), f"event {step}: snapshot {k} differs"
            assert guard_intact(new[k], n, elem_size) and guard_intact(new_snaps[k], n, elem_size)
            nb = ew.num_blocks(n * elem_size)
            assert np.array_equal(new_cks[k].cpu().numpy().view(np.uint64)[:nb], checksum.block_checksums(want[k]))
        shards = [t[:n] for t, n in zip(new, lens)]
        snaps = [t[:n] for t, n in zip(new_snaps, lens)]
        cks = [t[:ew.num_blocks(n * elem_size)] for t, n in zip(new_cks, lens)]
        dp = new_dp


def test_null_buffers_are_rejected():
    plan = ew.ew_plan(4, 3, 0b1011, 1 << 16, 4096)
    ew.ew_plan_upload(plan, 0, stream())
    old = [torch.zeros(plan.old_shard_len(j), dtype=torch.int32, device=DEV) for j in range(4)]
    stage = torch.zeros(plan.stage_len, dtype=torch.int32, device=DEV)
    with pytest.raises(ew.EwError) as e:   # rank 2 failed and no snapshot of it was passed
        ew.ew_pack(plan, old, [None] * 4, stage, 4, stream())
    assert e.value.code == ew.EW_EINVAL
    with pytest.raises(ew.EwError):
        ew.ew_pack(plan, old, [None, None, old[2], None], stage, 3, stream())
    with pytest.raises(ValueError):        # binding refuses a short arena before any launch
        ew.ew_pack(plan, old, [None, None, old[2], None], stage[:-8], 4, stream())
    # failed rank's live shard may be NULL: it is never read
    ew.ew_pack(plan, [old[0], old[1], None, old[3]], [None, None, old[2], None], stage, 4, stream())
    torch.cuda.synchronize()


def test_plain_copy_yardstick():
    rng = np.random.default_rng(5)
    for nbytes in (16, 4096, 4096 * 3 + 16, 5 * MIB + 160):
        raw = rng.integers(0, 256, nbytes, dtype=np.uint8)
        src = torch.from_numpy(raw).to(DEV)
        dst = torch.full((nbytes + 64,), 0x5A, dtype=torch.uint8, device=DEV)
        ew.ew_memcpy(src, dst, nbytes, stream())
        torch.cuda.synchronize()
        assert np.array_equal(dst[:nbytes].cpu().numpy(), raw) and bool((dst[nbytes:] == 0x5A).all())
    with pytest.raises(ew.EwError):
        ew.ew_memcpy(src, dst, 24, stream())


def test_snapshot_on_many_streams():
    """More streams than scratch regions: regions change hands (the new owner waits on the device
    for the previous use); every result is the oracle's."""
    rng = np.random.default_rng(77)
    streams = [torch.cuda.Stream() for _ in range(6)]
    nbytes = 5 * MIB + 4096 + 9
    raw = [rng.integers(0, 256, nbytes, dtype=np.uint8) for _ in streams]
    src = [torch.from_numpy(r).to(DEV) for r in raw]
    dst = [torch.zeros(nbytes, dtype=torch.uint8, device=DEV) for _ in streams]
    ck = [torch.zeros((ew.num_blocks(nbytes), 2), dtype=torch.int64, device=DEV) for _ in streams]
    torch.cuda.synchronize()
    for rep in range(3):
        for i, s in enumerate(streams):
            ew.ew_snapshot(src[i], dst[i], nbytes, ck[i], s.cuda_stream)
    torch.cuda.synchronize()
    for i in range(len(streams)):
        assert np.array_equal(dst[i].cpu().numpy(), raw[i])
        assert np.array_equal(ck[i].cpu().numpy().view(np.uint64), checksum.block_checksums(raw[i]))


def test_snapshot_on_the_per_thread_stream():
    """The per-thread default stream is one handle value for a different stream in every host
    thread, so it must never be taken for the owner of a scratch region: eight calls in a row on it
    (twice the number of regions) go through the event-ordered handover and give the oracle's result."""
    HIP_STREAM_PER_THREAD = 2
    rng = np.random.default_rng(78)
    nbytes = 3 * MIB + 100
    raw = [rng.integers(0, 256, nbytes, dtype=np.uint8) for _ in range(8)]
    src = [torch.from_numpy(r).to(DEV) for r in raw]
    dst = [torch.zeros(nbytes, dtype=torch.uint8, device=DEV) for _ in raw]
    ck = [torch.zeros((ew.num_blocks(nbytes), 2), dtype=torch.int64, device=DEV) for _ in raw]
    torch.cuda.synchronize()
    for i in range(len(raw)):
        ew.ew_snapshot(src[i], dst[i], nbytes, ck[i], HIP_STREAM_PER_THREAD)
    torch.cuda.synchronize()
    for i in range(len(raw)):
        assert np.array_equal(dst[i].cpu().numpy(), raw[i])
        assert np.array_equal(ck[i].cpu().numpy().view(np.uint64), checksum.block_checksums(raw[i]))


def test_snapshot_from_several_host_threads():
    """Six host threads, each with a stream of its own, issue snapshots at the same time (ctypes
    releases the interpreter lock during a call): more threads than scratch regions, so regions
    change hands while other threads are inside the library.  Every result is the oracle's."""
    import threading
    rng = np.random.default_rng(79)
    n_threads, reps = 6, 12
    nbytes = [2 * MIB + 4096 * i + 7 * i for i in range(n_threads)]
    raw = [rng.integers(0, 256, n, dtype=np.uint8) for n in nbytes]
    src = [torch.from_numpy(r).to(DEV) for r in raw]
    dst = [torch.zeros(n, dtype=torch.uint8, device=DEV) for n in nbytes]
    ck = [torch.zeros((ew.num_blocks(n), 2), dtype=torch.int64, device=DEV) for n in nbytes]
    streams = [torch.cuda.Stream() for _ in range(n_threads)]
    torch.cuda.synchronize()
    errors = []
    go = threading.Barrier(n_threads)

    def work(i):
        try:
            go.wait()
            for _ in range(reps):
                ew.ew_snapshot(src[i], dst[i], nbytes[i], ck[i], streams[i].cuda_stream)
        except Exception as e:   # reported by the main thread
            errors.append((i, repr(e)))

    threads = [threading.Thread(target=work, args=(i,)) for i in range(n_threads)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for i in range(n_threads):
        assert np.array_equal(dst[i].cpu().numpy(), raw[i])
        assert np.array_equal(ck[i].cpu().numpy().view(np.uint64), checksum.block_checksums(raw[i]))


def test_two_host_threads_share_one_stream():
    """Two host threads issue snapshots on the SAME stream at the same time.  Their (slot kernel, fold
    kernel) pairs may interleave on the stream, so each call holds a scratch region of its own while it
    enqueues; every result is the oracle's."""
    import threading
    rng = np.random.default_rng(80)
    n_threads, reps = 2, 40
    nbytes = [3 * MIB + 4096 + 9, 2 * MIB + 8192 + 3]
    raw = [[rng.integers(0, 256, nbytes[i], dtype=np.uint8) for _ in range(3)] for i in range(n_threads)]
    src = [[torch.from_numpy(r).to(DEV) for r in rs] for rs in raw]
    dst = [[torch.zeros(nbytes[i], dtype=torch.uint8, device=DEV) for _ in range(3)] for i in range(n_threads)]
    ck = [[torch.zeros((ew.num_blocks(nbytes[i]), 2), dtype=torch.int64, device=DEV) for _ in range(3)]
          for i in range(n_threads)]
    shared = torch.cuda.Stream()
    torch.cuda.synchronize()
    errors = []
    go = threading.Barrier(n_threads)

    def work(i):
        try:
            go.wait()
            for r in range(reps):
                b = r % 3
                ew.ew_snapshot(src[i][b], dst[i][b], nbytes[i], ck[i][b], shared.cuda_stream)
        except Exception as e:   # reported by the main thread
            errors.append((i, repr(e)))

    threads = [threading.Thread(target=work, args=(i,)) for i in range(n_threads)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for i in range(n_threads):
        for b in range(3):
            assert np.array_equal(dst[i][b].cpu().numpy(), raw[i][b])
            assert np.array_equal(ck[i][b].cpu().numpy().view(np.uint64), checksum.block_checksums(raw[i][b]))


def test_enqueues_on_two_streams_overlap():
    """The scratch lock is held only while a region is picked and while its event is recorded, so two
    host threads on two streams are inside the library's enqueue section at the same time: the
    library's own count of regions held at once reaches two (tried a few times: whether the two
    threads meet in a given round is up to the scheduler), and the results are the oracle's."""
    import threading
    rng = np.random.default_rng(81)
    ew.ew_set_param("snapshot_wave_min_bytes", 0)   # one slot per KiB: a region covers 2 GiB, so ...
    nbytes = 5 * (1 << 30) // 2 + 4096 + 5     # ... 2.5 GiB takes two passes (four launches) per call
    raw8 = rng.integers(0, 1 << 62, 1 << 16, dtype=np.int64)
    src = torch.from_numpy(raw8).to(DEV).repeat((nbytes + 8 * len(raw8) - 1) // (8 * len(raw8))).view(torch.uint8)[:nbytes]
    dst = [torch.zeros(nbytes, dtype=torch.uint8, device=DEV) for _ in range(2)]
    ck = [torch.zeros((ew.num_blocks(nbytes), 2), dtype=torch.int64, device=DEV) for _ in range(2)]
    streams = [torch.cuda.Stream() for _ in range(2)]
    torch.cuda.synchronize()
    errors = []
    seen = 0
    for attempt in range(12):
        ew.ew_set_param("scratch_max_concurrent", 0)
        go = threading.Barrier(2)

        def work(i):
            try:
                go.wait()
                for _ in range(60):
                    ew.ew_snapshot(src, dst[i], nbytes, ck[i], streams[i].cuda_stream)
            except Exception as e:   # reported by the main thread
                errors.append((i, repr(e)))

        threads = [threading.Thread(target=work, args=(i,)) for i in range(2)]
        for t in threads:
            t.start()
        for t in threads:
            t.join()
        torch.cuda.synchronize()
        assert not errors, errors
        seen = ew.ew_get_param("scratch_max_concurrent")
        if seen >= 2:
            break
    assert seen >= 2, "two streams' enqueues never overlapped"
    want = None
    for i in range(2):
        assert torch.equal(dst[i], src)
        got = ck[i].cpu().numpy().view(np.uint64)
        if want is None:   # oracle on sampled blocks (both ends, both sides of the pass boundary), then equality
            for b in (0, 1, 2047, 2048, 2049, len(got) - 2, len(got) - 1):
                host = src[b * MIB:min((b + 1) * MIB, nbytes)].cpu().numpy()
                assert np.array_equal(got[b], checksum.block_checksums(host)[0]), f"block {b}"
            want = got
        assert np.array_equal(got, want)


@pytest.mark.timeout(600)
def test_snapshot_longer_than_one_scratch_pass():
    """17 GiB + ragged tail: nine passes over a scratch region, whose slots cover 2 GiB."""
    nbytes = 17 * (1 << 30) + 3 * MIB + 4096 + 5
    src = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    g = torch.Generator(device=DEV)
    g.manual_seed(11)
    v = src[: (nbytes // 8) * 8].view(torch.int64)
    step = 1 << 27
    for o in range(0, v.numel(), step):
        n = min(step, v.numel() - o)
        v[o:o + n] = torch.randint(-(1 << 62), 1 << 62, (n,), dtype=torch.int64, device=DEV, generator=g)
    src[(nbytes // 8) * 8:] = 0xA7
    dst = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
    nb = ew.num_blocks(nbytes)
    ck = torch.full((nb, 2), -1, dtype=torch.int64, device=DEV)
    ew.ew_snapshot(src, dst, nbytes, ck, stream())
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    got = ck.cpu().numpy().view(np.uint64)
    # oracle on sampled blocks incl. both sides of every pass boundary and the ragged last block
    blocks = sorted({0, 1, 2047, 2048, 2049, 4095, 4096, 8191, 8192, 8193, 16383, 16384, 16385, nb - 2, nb - 1}
                    | set(np.random.default_rng(1).integers(0, nb, 24).tolist()))
    for b in blocks:
        host = src[b * MIB:min((b + 1) * MIB, nbytes)].cpu().numpy()
        assert np.array_equal(got[b], checksum.block_checksums(host)[0]), f"block {b}"
    # every block: sum of the records equals torch's wrapping sum of all words
    total = int(v.sum().item()) & ((1 << 64) - 1)
    tail = int.from_bytes(bytes([0xA7] * (nbytes % 8)), "little")
    assert (int(got[:, 0].sum(dtype=np.uint64)) & ((1 << 64) - 1)) == (total + tail) & ((1 << 64) - 1)


def test_fused_unpack_on_many_streams():
    """Six streams take turns with four scratch regions; each stream's result is the oracle's."""
    rng = np.random.default_rng(123)
    Do, Dn, mask, N, C, es = 5, 4, 0b11011, 1_200_000, 40_000, 4
    starts = layout.unit_starts(N, C)
    alive = layout.alive_list(Do, mask)
    lens = layout.shard_lengths(starts, Do)
    plan = ew.ew_plan(Do, Dn, mask, N, C)
    ew.ew_plan_upload(plan, 0, stream())
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in range(6)]
    jobs = []
    for s in streams:
        data = random_shards(lens, es, rng)
        want = layout.reshard([d if alive[j] else None for j, d in enumerate(data)],
                              [None if alive[j] else d for j, d in enumerate(data)], Do, Dn, mask, starts)
        old = [to_dev(d, es) if alive[j] else None for j, d in enumerate(data)]
        snaps = [None if alive[j] else to_dev(d, es) for j, d in enumerate(data)]
        stage = torch.zeros(plan.stage_len, dtype=torch.int32, device=DEV)
        new = [torch.zeros(plan.new_shard_len(k), dtype=torch.int32, device=DEV) for k in range(Dn)]
        nsn = [torch.zeros_like(t) for t in new]
        ck = [torch.zeros((ew.num_blocks(t.numel() * es), 2), dtype=torch.int64, device=DEV) for t in new]
        jobs.append((s, old, snaps, stage, new, nsn, ck, want))
    torch.cuda.synchronize()
    for rep in range(3):
        for (s, old, snaps, stage, new, nsn, ck, want) in jobs:
            ew.ew_pack(plan, old, snaps, stage, es, s.cuda_stream)
            ew.ew_unpack_snapshot(plan, stage, old, snaps, new, nsn, ck, es, s.cuda_stream)
    torch.cuda.synchronize()
    for (s, old, snaps, stage, new, nsn, ck, want) in jobs:
        for k in range(Dn):
            assert np.array_equal(np_bits(new[k]), want[k]) and np.array_equal(np_bits(nsn[k]), want[k])
            assert np.array_equal(ck[k].cpu().numpy().view(np.uint64), checksum.block_checksums(want[k]))
    plan.close()
