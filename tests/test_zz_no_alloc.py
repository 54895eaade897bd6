"""ew_snapshot_noalloc, the entry point for callers that cannot allocate (its checksum slots live in
a fixed device array): through the C ABI against ew_snapshot's output and the CPU oracle, bit for
bit, on two calls in a row of which the second is smaller, so that whatever the first call left in
the array would show if it leaked into the second."""
import numpy as np
import pytest
import torch

import paper_2510_00606_amd as ew
from oracle import checksum

from gpu_util import DEV, stream

pytestmark = pytest.mark.gpu

MIB = 1 << 20


@pytest.fixture(autouse=True)
def default_shape():
    saved = ew.ew_get_param("snapshot_wave_min_bytes")
    yield
    ew.ew_set_param("snapshot_wave_min_bytes", saved)


def both_entry_points(nbytes, seed, shift=0):
    """Runs ew_snapshot_noalloc and ew_snapshot on the same seeded bytes; returns nothing, asserts."""
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    n8 = (nbytes + shift + 15) // 8 + 2
    src_all = torch.randint(-(1 << 62), 1 << 62, (n8,), dtype=torch.int64, device=DEV, generator=g).view(torch.uint8)
    src = src_all[shift:shift + nbytes]
    nb = ew.num_blocks(nbytes)
    out = {}
    for name, fn in (("noalloc", ew.ew_snapshot_noalloc), ("snapshot", ew.ew_snapshot)):
        dst_all = torch.full((nbytes + shift + 64,), 0x5A, dtype=torch.uint8, device=DEV)
        dst = dst_all[shift:shift + nbytes]
        ck = torch.full((nb + 1, 2), -1, dtype=torch.int64, device=DEV)
        fn(src, dst, nbytes, ck, stream())
        torch.cuda.synchronize()
        assert bool((dst_all[:shift] == 0x5A).all()) and bool((dst_all[shift + nbytes:] == 0x5A).all()), name
        out[name] = (dst, ck)
    assert torch.equal(out["noalloc"][0], src), "allocation-free snapshot bytes differ from the source"
    assert torch.equal(out["noalloc"][0], out["snapshot"][0])
    assert torch.equal(out["noalloc"][1], out["snapshot"][1]), "checksums differ from ew_snapshot's"
    got = out["noalloc"][1].cpu().numpy().view(np.uint64)
    assert np.array_equal(got[:nb], checksum.block_checksums(src.cpu().numpy())), "checksums differ from the oracle's"
    assert (got[nb] == np.uint64((1 << 64) - 1)).all(), "record past the end was written"


@pytest.mark.parametrize("wave_min", [1 << 62, 0])     # 256-lane workgroups (the default) / one-wave workgroups
def test_two_calls_in_a_row_second_smaller(wave_min):
    ew.ew_set_param("snapshot_wave_min_bytes", wave_min)
    both_entry_points(300 * MIB + 3 * 4096 + 5, 1)     # ragged tail; 77 k slots (307 k with one-wave workgroups)
    both_entry_points(37 * MIB + 1024 + 9, 2)          # far fewer slots: what the first call left must not leak in
    both_entry_points(MIB + 16, 3)
    both_entry_points(5, 4)


def test_largest_size_then_a_small_one():
    ew.ew_set_param("snapshot_wave_min_bytes", 0)      # one slot per KiB: every slot of the array in use
    both_entry_points(ew.EW_NOALLOC_MAX_BYTES, 5)
    both_entry_points(2 * MIB - 8, 6)
    ew.ew_set_param("snapshot_wave_min_bytes", 1 << 62)
    both_entry_points(ew.EW_NOALLOC_MAX_BYTES, 7)
    both_entry_points(3 * MIB + 40, 8)


def test_unaligned_buffers_take_the_scratch_free_kernel():
    both_entry_points(2 * MIB + 77, 7, shift=3)
    both_entry_points(4097, 8, shift=8)


def test_too_big_is_refused_and_nothing_is_written():
    src = torch.zeros(64, dtype=torch.uint8, device=DEV)
    dst = torch.full((64,), 0x5A, dtype=torch.uint8, device=DEV)
    ck = torch.full((1, 2), -1, dtype=torch.int64, device=DEV)
    with pytest.raises(ew.EwError) as e:   # raw addresses: the binding's own size checks do not apply
        ew.ew_snapshot_noalloc(src.data_ptr(), dst.data_ptr(), ew.EW_NOALLOC_MAX_BYTES + 1, ck.data_ptr(), stream())
    assert e.value.code == ew.EW_ETOOBIG and "too big" in str(e.value)
    torch.cuda.synchronize()
    assert bool((dst == 0x5A).all()) and bool((ck == -1).all())
    ew.ew_snapshot_noalloc(src, dst, 0, ck, stream())   # nothing to do
    torch.cuda.synchronize()
    assert bool((dst == 0x5A).all()) and bool((ck == -1).all())


def test_on_a_second_stream_after_the_first():
    """Calls on different streams share the one array, so the caller orders them; ordered, they agree."""
    side = torch.cuda.Stream()
    both_entry_points(9 * MIB + 40, 9)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        both_entry_points(6 * MIB + 24, 10)
    side.synchronize()
