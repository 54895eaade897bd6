"""Helpers for the GPU parity tests: device state built from seeded inputs, calls through the
C-ABI binding, host copies for the oracle.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

import paper_2510_00606_amd as ew
from paper_2510_00606_amd import synth

DEV = "cuda:0"
GUARD = 64  # sentinel elements after every output buffer


def stream():
    return torch.cuda.current_stream().cuda_stream


def np_bits(t):
    return synth.to_numpy_bits(t)


def int_dtype(elem_size):
    return {2: torch.int16, 4: torch.int32}[elem_size]


def random_shards(lengths, elem_size, rng):
    """Host numpy arrays of random bits, one per rank."""
    npdt = {2: np.uint16, 4: np.uint32}[elem_size]
    return [rng.integers(0, 1 << (8 * elem_size), size=n, dtype=np.uint64).astype(npdt) for n in lengths]


def to_dev(a: np.ndarray, elem_size):
    t = torch.from_numpy(a.view({2: np.int16, 4: np.int32}[elem_size]).copy())
    return t.to(DEV)


def guarded(n, elem_size, fill=0x5A):
    """Output buffer of n elements followed by GUARD sentinel elements."""
    t = torch.full((n + GUARD,), fill | (fill << 8) if elem_size == 2 else 0x5A5A5A5A, dtype=int_dtype(elem_size),
                   device=DEV)
    return t


def guard_intact(t, n, elem_size):
    want = 0x5A5A if elem_size == 2 else 0x5A5A5A5A
    return bool((t[n:] == want).all())


def run_reshard(plan, old_dev, snap_dev, elem_size, tile_elems=0):
    """pack + unpack through the C ABI; returns (stage tensor, list of new-shard tensors)."""
    ew.ew_plan_upload(plan, tile_elems, stream())
    stage = guarded(plan.stage_len, elem_size)
    new = [guarded(plan.new_shard_len(k), elem_size) for k in range(plan.new_dp)]
    ew.ew_pack(plan, old_dev, snap_dev, stage, elem_size, stream())
    ew.ew_unpack(plan, stage, old_dev, snap_dev, new, elem_size, stream())
    torch.cuda.synchronize()
    return stage, new
