"""The five named workloads at full size on the GPU, in the launch configuration bench.py times
(library defaults), against the CPU oracle.

  tiny, 7b_stage      every array compared element by element with the oracle's result
  7b_rank_snapshot    snapshot bytes + every checksum record against the oracle; one flipped bit
                      must be located (block index and bit lane)
  13b_stage           every array compared element by element with the oracle's result
  70b_stage           every array (17 GB of bf16, 34 GB per fp32 array) compared element by element
                      with the oracle's result, a window of whole units (about 1 GiB of state) at a
                      time: the oracle reshards the window's slice of every old shard, regenerated
                      from the seeded generator, and the result is compared with the same slice
                      of every new shard; the oracle's checksums are taken over its own result as
                      the windows stream by and compared record by record with the fused call's
In addition, for every array of every workload: sampled elements of every new shard (incl. both
ends) are recomputed one by one by the oracle's locator from the seeded generator, and the multiset
of 64-bit words is shown to be conserved (wrapping sums of w and w*w, torch integer ops).
Every workload also runs the fused ew_unpack_snapshot: new shards and snapshot copies equal the
verified result, every checksum record equals the oracle's; and the arena-free ew_reshard /
ew_reshard_snapshot, whose outputs must equal those verified ones.
"""
import gc

import numpy as np
import pytest
import torch

import paper_2510_00606_amd as ew
from oracle import checksum, layout
from paper_2510_00606_amd import configs, synth

from gpu_util import DEV, stream

pytestmark = pytest.mark.gpu


def free():
    gc.collect()
    torch.cuda.empty_cache()


def word_moments(tensors):
    """Wrapping sums of the 64-bit words and of their squares over a list of device tensors."""
    s1 = s2 = 0
    for t in tensors:
        if t.numel() == 0:
            continue
        w = t.view(torch.int64)
        s1 = (s1 + int(w.sum().item())) & ((1 << 64) - 1)
        s2 = (s2 + int((w * w).sum().item())) & ((1 << 64) - 1)
    return s1, s2


class Pinned:
    """One page-locked host buffer, reused for every device-to-host copy of a windowed comparison."""

    def __init__(self, nbytes):
        self.buf = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
        self.used = 0

    def reset(self):
        self.used = 0

    def fetch(self, t):
        """Host copy of device tensor t as unsigned integers of its element width (a view of the
        buffer: valid until reset())."""
        n = t.numel() * t.element_size()
        off = (self.used + 63) & ~63
        assert off + n <= self.buf.numel()
        self.buf[off:off + n].copy_(t.contiguous().view(torch.uint8))
        self.used = off + n
        torch.cuda.synchronize()
        return self.buf[off:off + n].numpy().view({2: np.uint16, 4: np.uint32}[t.element_size()])


def windowed_oracle_compare(w, arr, starts, new, fused_cksums, window_elems=1 << 28):
    """Every element of every new shard in `new` (device tensors), and every record of
    `fused_cksums` (device, one array per new rank), against the CPU oracle, streaming: units
    [u0, u1) of the flat state occupy one contiguous slice of every old and of every new shard, so
    the oracle reshards window after window.  Its inputs are regenerated from the seeded generator
    (never read back from buffers the library has touched); its checksums are taken over its own
    result, carried across windows up to whole 1 MiB blocks."""
    es = synth.ELEM_SIZE[arr]
    Do, Dn = w.old_dp, w.new_dp
    alive = layout.alive_list(Do, w.alive_mask)
    n_units = len(starts) - 1
    o_off, n_off = [0] * Do, [0] * Dn
    pend = [np.empty(0, np.uint8) for _ in range(Dn)]
    blk = [0] * Dn
    cks = [c.cpu().numpy().view(np.uint64) for c in fused_cksums]
    pin = Pinned(2 * (window_elems + int(np.diff(starts).max())) * es + 64 * (Do + 2))
    u0 = 0
    while u0 < n_units:
        u1 = u0 + 1
        while u1 < n_units and int(starts[u1 + 1] - starts[u0]) <= window_elems:
            u1 += 1
        ws = (starts[u0:u1 + 1] - starts[u0]).astype(np.int64)
        ol, nl = layout.shard_lengths(ws, Do), layout.shard_lengths(ws, Dn)
        pin.reset()
        host = [pin.fetch(synth.fill(w.seed, j, arr, o_off[j], ol[j], DEV)) for j in range(Do)]
        want = layout.reshard([h if alive[j] else None for j, h in enumerate(host)],
                              [None if alive[j] else h for j, h in enumerate(host)], Do, Dn, w.alive_mask, ws)
        mark = pin.used
        for k in range(Dn):
            pin.used = mark
            got = pin.fetch(new[k][n_off[k]:n_off[k] + nl[k]])
            assert np.array_equal(got, want[k]), f"{w.name} {arr}: new shard {k}, units {u0}..{u1 - 1} differ"
            pend[k] = np.concatenate([pend[k], want[k].view(np.uint8)])
            full = len(pend[k]) >> 20
            if full:
                rec = checksum.block_checksums(pend[k][:full << 20])
                assert np.array_equal(cks[k][blk[k]:blk[k] + full], rec), \
                    f"{w.name} {arr}: fused checksums of rank {k}, blocks {blk[k]}..{blk[k] + full - 1}"
                blk[k] += full
                pend[k] = pend[k][full << 20:].copy()
        o_off = [a + b for a, b in zip(o_off, ol)]
        n_off = [a + b for a, b in zip(n_off, nl)]
        print(f"[{w.name}] {arr}: units {u0}..{u1 - 1} of {n_units} equal the oracle's", flush=True)
        u0 = u1
    for k in range(Dn):
        if len(pend[k]):
            assert np.array_equal(cks[k][blk[k]:blk[k] + 1], checksum.block_checksums(pend[k])), \
                f"{w.name} {arr}: last checksum record of rank {k}"
            blk[k] += 1
        assert blk[k] == len(cks[k]) and n_off[k] == new[k].numel()
    del pin


def run_workload_array(w, arr, plan, starts, full_compare, snapshot_all):
    es = synth.ELEM_SIZE[arr]
    alive = layout.alive_list(w.old_dp, w.alive_mask)
    st = stream()
    old = [synth.fill(w.seed, j, arr, 0, plan.old_shard_len(j), DEV) for j in range(w.old_dp)]
    # per-step snapshot (ring placement: the copy of rank j's partition lives with rank j-1)
    snaps, sums = [None] * w.old_dp, [None] * w.old_dp
    for j in range(w.old_dp):
        if snapshot_all or not alive[j]:
            nbytes = old[j].numel() * es
            snaps[j] = torch.empty_like(old[j])
            sums[j] = torch.zeros((ew.num_blocks(nbytes), 2), dtype=torch.int64, device=DEV)
            ew.ew_snapshot(old[j], snaps[j], nbytes, sums[j], st)
    torch.cuda.synchronize()
    host_old = [synth.to_numpy_bits(t) for t in old] if full_compare else None
    src_moments = word_moments(old)
    # failure: the device memory of failed ranks is gone
    for j in w.failed:
        old[j].view(torch.uint8).fill_(0xFF)
    # integrity check of the snapshots that will be read
    for j in w.failed:
        nbytes = snaps[j].numel() * es
        got = torch.zeros_like(sums[j])
        n_bad = torch.zeros(1, dtype=torch.int64, device=DEV)
        bad = torch.zeros(8, dtype=torch.int64, device=DEV)
        diffs = torch.zeros((8, 2), dtype=torch.int64, device=DEV)
        ew.ew_verify(snaps[j], nbytes, sums[j], got, n_bad, bad, diffs, 8, st)
        assert int(n_bad.item()) == 0
    stage = torch.empty(plan.stage_len, dtype=old[0].dtype, device=DEV)
    new = [torch.empty(plan.new_shard_len(k), dtype=old[0].dtype, device=DEV) for k in range(w.new_dp)]
    for t in new:
        t.view(torch.uint8).fill_(0x5A)
    ew.ew_pack(plan, old, snaps, stage, es, st)
    ew.ew_unpack(plan, stage, old, snaps, new, es, st)
    torch.cuda.synchronize()

    # (1) the multiset of words is conserved
    assert word_moments(new) == src_moments
    # (2) sampled elements, recomputed one by one from the generator through the oracle's locator
    rng = np.random.default_rng([w.seed, synth.ARRAYS.index(arr)])
    for k in range(w.new_dp):
        n = plan.new_shard_len(k)
        offs = np.unique(np.concatenate([np.arange(min(n, 64)), np.arange(max(0, n - 64), n),
                                         rng.integers(0, n, 1 << 16)]))
        _, owner, ooff = layout.locate_new_elements(starts, w.old_dp, w.new_dp, k, offs)
        want = np.empty(len(offs), dtype={2: np.uint16, 4: np.uint32}[es])
        for j in range(w.old_dp):
            m = owner == j
            if m.any():
                want[m] = synth.to_numpy_bits(synth.values_at(w.seed, j, arr, torch.from_numpy(ooff[m])))
        got = synth.to_numpy_bits(new[k][torch.from_numpy(offs).to(DEV)])
        assert np.array_equal(got, want), f"{w.name} {arr}: sampled elements of new shard {k} differ"
    # (3) everything, element by element
    want_new = None
    if full_compare:
        o_sh = [h if alive[j] else None for j, h in enumerate(host_old)]
        o_sn = [None if alive[j] else h for j, h in enumerate(host_old)]
        flat = layout.reconstruct_flat(o_sh, o_sn, w.old_dp, alive, starts)
        want_new = layout.slice_flat(flat, w.new_dp, starts)
        for k in range(w.new_dp):
            assert np.array_equal(synth.to_numpy_bits(new[k]), want_new[k]), f"{w.name} {arr}: new shard {k} differs"
        del flat

    # (4) the fused form: same new shards, snapshot copies equal to them, checksums = the oracle's
    new2 = [torch.empty_like(t) for t in new]
    snap2 = [torch.empty_like(t) for t in new]
    for t in new2 + snap2:
        t.view(torch.uint8).fill_(0xA5)
    ck2 = [torch.full((ew.num_blocks(t.numel() * es), 2), -1, dtype=torch.int64, device=DEV) for t in new]
    ew.ew_unpack_snapshot(plan, stage, old, snaps, new2, snap2, ck2, es, st)
    torch.cuda.synchronize()
    rng = np.random.default_rng([w.seed, 7, synth.ARRAYS.index(arr)])
    for k in range(w.new_dp):
        view = torch.int16 if es == 2 else torch.int32
        assert torch.equal(new2[k].view(view), new[k].view(view)), f"{w.name} {arr}: fused new shard {k} differs"
        assert torch.equal(snap2[k].view(view), new[k].view(view)), f"{w.name} {arr}: fused snapshot {k} differs"
        got = ck2[k].cpu().numpy().view(np.uint64)
        nb = got.shape[0]
        if want_new is not None:
            assert np.array_equal(got, checksum.block_checksums(want_new[k])), f"{w.name} {arr}: fused checksums {k}"
    if want_new is None:
        # too large for one host copy: every element of `new` and every record of ck2 against the
        # oracle, window by window (new2 and snap2 were shown equal to `new` just above)
        windowed_oracle_compare(w, arr, starts, new, ck2)
    # (5) without the arena: every segment straight from its source, alone and fused with the snapshot
    for t in new2 + snap2:
        t.view(torch.uint8).fill_(0x3C)
    ew.ew_reshard(plan, old, snaps, new2, es, st)
    torch.cuda.synchronize()
    view = torch.int16 if es == 2 else torch.int32
    for k in range(w.new_dp):
        assert torch.equal(new2[k].view(view), new[k].view(view)), f"{w.name} {arr}: direct new shard {k} differs"
        new2[k].view(torch.uint8).fill_(0x3C)
    ck3 = [torch.full_like(c, -1) for c in ck2]
    ew.ew_reshard_snapshot(plan, old, snaps, new2, snap2, ck3, es, st)
    torch.cuda.synchronize()
    for k in range(w.new_dp):
        assert torch.equal(new2[k].view(view), new[k].view(view)) and torch.equal(snap2[k].view(view), new[k].view(view))
        assert torch.equal(ck3[k], ck2[k]), f"{w.name} {arr}: direct fused checksums of rank {k} differ"
    del old, snaps, stage, new, new2, snap2, want_new
    free()


def run_workload(name, full_arrays, snapshot_all):
    w = configs.ALL[name]()
    starts = w.unit_starts()
    plan = ew.ew_plan_bounds(w.old_dp, w.new_dp, w.alive_mask, starts)
    ew.ew_plan_upload(plan, 0, stream())
    s64 = starts.astype(np.int64)
    for arr in synth.ARRAYS:
        print(f"[{name}] array {arr}", flush=True)
        run_workload_array(w, arr, plan, s64, arr in full_arrays, snapshot_all)
    plan.close()


def test_tiny_all_arrays():
    run_workload("tiny", synth.ARRAYS, True)


@pytest.mark.timeout(900)
def test_7b_stage_all_arrays():
    run_workload("7b_stage", synth.ARRAYS, True)


@pytest.mark.timeout(900)
def test_13b_stage():
    run_workload("13b_stage", synth.ARRAYS, True)


@pytest.mark.timeout(1500)
def test_70b_stage():
    run_workload("70b_stage", (), False)


@pytest.mark.timeout(600)
def test_7b_rank_snapshot_and_bit_flip():
    w = configs.snapshot_7b()
    rng = np.random.default_rng([w.seed, 99])
    flip_arr = synth.ARRAYS[int(rng.integers(0, 4))]
    st = stream()
    for arr in synth.ARRAYS:
        es = synth.ELEM_SIZE[arr]
        nbytes = w.numel * es
        src = synth.fill(w.seed, 0, arr, 0, w.numel, DEV)
        snap = torch.empty_like(src)
        nb = ew.num_blocks(nbytes)
        assert nb == {2: 418, 4: 835}[es]
        sums = torch.zeros((nb, 2), dtype=torch.int64, device=DEV)
        ew.ew_snapshot(src, snap, nbytes, sums, st)
        torch.cuda.synchronize()
        assert torch.equal(src.view(torch.int16), snap.view(torch.int16))
        host = synth.to_numpy_bits(src)
        want = checksum.block_checksums(host)
        assert np.array_equal(sums.cpu().numpy().view(np.uint64), want)
        if arr == flip_arr:
            o, bit = int(rng.integers(0, nbytes)), int(rng.integers(0, 8))
            snap.view(torch.uint8)[o] ^= (1 << bit)
            got = torch.zeros_like(sums)
            n_bad = torch.zeros(1, dtype=torch.int64, device=DEV)
            bad = torch.full((4,), -1, dtype=torch.int64, device=DEV)
            diffs = torch.zeros((4, 2), dtype=torch.int64, device=DEV)
            ew.ew_verify(snap, nbytes, sums, got, n_bad, bad, diffs, 4, st)
            torch.cuda.synchronize()
            assert int(n_bad.item()) == 1
            assert int(bad[0].item()) == o >> 20
            d = diffs.cpu().numpy().view(np.uint64)[0]
            assert int(d[1]) == 1 << (8 * (o % 8) + bit)          # bit lane inside the 64-bit word
            hb = host.view(np.uint8).copy()
            hb[o] ^= np.uint8(1 << bit)
            o_bad, o_diffs = checksum.verify(hb, want)
            assert o_bad.tolist() == [o >> 20] and np.array_equal(o_diffs[0], d)
            lane, direction = ew.ew_single_bit_flip(int(d[0]), int(d[1]))   # "locate": block above, bit lane here
            assert lane == 8 * (o % 8) + bit and direction == (1 if (hb[o] >> bit) & 1 or lane == 63 else -1)
        del src, snap
        free()
