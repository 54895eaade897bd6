"""Interleaved ZeRO layout, flat-state reconstruction and re-slicing (CPU oracle).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Plain numpy, no blocking,
no segment tables: the reshard result is *defined* as

    new shards = slice( reconstruct(old shards, snapshots), new layout )

because the change of ZeRO layout is purely a change of ownership (Sec. 6.3,
last paragraph): the logical flat state is the same before and after.

Notation follows the paper: D = DP degree, O_i^j = rank j's piece of unit
("layer") i, F = failed set, worker i holds the snapshot of worker (i+1) mod n.

Readings taken where the paper is silent (each is restated in the repo's
design notes):
  * unit = the paper's "layer": a run of consecutive elements of the flat
    state given by explicit boundaries (uniform `chunk`, last unit short).
  * a unit whose length the DP degree does not divide: boundaries are the floor split
    of the unit's 8-element granules, b_j = min(L, 8*floor(j*ceil(L/8)/D)).
  * survivors keep their relative order and are renumbered densely from 0;
    joiners are appended; if fewer new ranks than survivors, the highest
    survivors only give data away.
  * an alive rank's data always comes from its live shard; a failed rank's
    data comes from the snapshot held by its ring predecessor.
"""
from __future__ import annotations

import numpy as np

GRANULE = 8  # elements: 16 B of bf16, 32 B of fp32


class Unrecoverable(Exception):
    """A failed rank's ring predecessor failed too (Sec. 5.2, step 1)."""


# --------------------------------------------------------------------------
# layout definition (Sec. 6.3 "Interleaved Assignment", Fig. 10b)
# --------------------------------------------------------------------------
def piece_bounds(L: int, D: int) -> list[int]:
    """Boundaries b_0..b_D of one unit of L elements split over D ranks.

    Rank j owns [b_j, b_{j+1}) of the unit.  Every rank owns a piece of every
    unit: its shard number j of each of them (Sec. 6.3, Fig. 10b).
    """
    if D < 1 or L < 0:
        raise ValueError("bad unit/degree")
    n_gran = -(-L // GRANULE)
    return [min(L, GRANULE * ((j * n_gran) // D)) for j in range(D + 1)]


def unit_starts(numel: int, chunk: int) -> np.ndarray:
    """Unit boundaries for a fixed interleave chunk: 0, C, 2C, ..., numel."""
    if chunk < 1 or numel < 0:
        raise ValueError("bad numel/chunk")
    s = list(range(0, numel, chunk)) + [numel]
    return np.asarray(s, dtype=np.int64)


def shard_lengths(starts: np.ndarray, D: int) -> list[int]:
    """Length of each rank's shard = sum over units of its piece length."""
    out = [0] * D
    for u in range(len(starts) - 1):
        b = piece_bounds(int(starts[u + 1] - starts[u]), D)
        for j in range(D):
            out[j] += b[j + 1] - b[j]
    return out


# --------------------------------------------------------------------------
# membership (Sec. 5.1 ring placement; Sec. 5.2 step 1 "Integrity Check")
# --------------------------------------------------------------------------
def alive_list(old_dp: int, alive_mask: int) -> list[bool]:
    if alive_mask >> old_dp:
        raise ValueError("alive_mask has bits above old_dp")
    return [bool((alive_mask >> j) & 1) for j in range(old_dp)]


def holder_of(owner: int, old_dp: int, alive: list[bool]) -> int:
    """Old rank that physically has `owner`'s shard: itself if alive, else its
    ring predecessor, which keeps the snapshot of worker (i+1) mod n."""
    if alive[owner]:
        return owner
    h = (owner - 1) % old_dp
    if not alive[h]:
        raise Unrecoverable(f"rank {owner} and its snapshot holder {h} both failed")
    return h


def check_recoverable(old_dp: int, alive: list[bool]) -> None:
    if not any(alive):
        raise Unrecoverable("no survivor")
    for j in range(old_dp):
        holder_of(j, old_dp, alive)


def new_rank_of(old_dp: int, new_dp: int, alive: list[bool]) -> list[int]:
    """Old rank -> new rank (-1 for failed ranks and for survivors that leave)."""
    out, nxt = [], 0
    for j in range(old_dp):
        if alive[j] and nxt < new_dp:
            out.append(nxt)
            nxt += 1
        else:
            out.append(-1)
    return out


# --------------------------------------------------------------------------
# reconstruct -> slice  (Sec. 5.2 steps 2-4; Sec. 6.3 last paragraph)
# --------------------------------------------------------------------------
def reconstruct_flat(old_shards, snapshots, old_dp, alive, starts):
    """Logical flat array that standard ZeRO would all-gather from the old
    layout.  old_shards[j] is rank j's live shard (ignored when j failed);
    snapshots[j] is the snapshot OF owner j's shard (read only when j failed).
    """
    check_recoverable(old_dp, alive)
    src = []
    for j in range(old_dp):
        a = old_shards[j] if alive[j] else snapshots[j]
        if a is None:
            raise ValueError(f"no data for old rank {j}")
        src.append(np.asarray(a))
    numel = int(starts[-1])
    flat = np.empty(numel, dtype=src[0].dtype)
    cur = [0] * old_dp
    for u in range(len(starts) - 1):
        s = int(starts[u])
        b = piece_bounds(int(starts[u + 1]) - s, old_dp)
        for j in range(old_dp):
            n = b[j + 1] - b[j]
            flat[s + b[j]:s + b[j + 1]] = src[j][cur[j]:cur[j] + n]
            cur[j] += n
    for j in range(old_dp):
        if cur[j] != len(src[j]):
            raise ValueError(f"old shard {j} has {len(src[j])} elements, layout says {cur[j]}")
    return flat


def slice_flat(flat, new_dp, starts):
    """Cut the flat array into new_dp shards under the interleaved layout."""
    flat = np.asarray(flat)
    parts = [[] for _ in range(new_dp)]
    for u in range(len(starts) - 1):
        s = int(starts[u])
        b = piece_bounds(int(starts[u + 1]) - s, new_dp)
        for k in range(new_dp):
            parts[k].append(flat[s + b[k]:s + b[k + 1]])
    return [np.concatenate(p) if p else flat[:0].copy() for p in parts]


def reshard(old_shards, snapshots, old_dp, new_dp, alive_mask, starts):
    """New shards after a DP change old_dp -> new_dp with the given survivors."""
    alive = alive_list(old_dp, alive_mask)
    flat = reconstruct_flat(old_shards, snapshots, old_dp, alive, starts)
    return slice_flat(flat, new_dp, starts)


# --------------------------------------------------------------------------
# what travels: per-(holder -> destination) messages (Fig. 7b, M_overlap)
# --------------------------------------------------------------------------
def held_ranges(u_len: int, h: int, old_dp: int, alive: list[bool]):
    """Element ranges of one unit that old rank h can serve, ascending:
    its own piece (live) and, if its ring successor failed, that piece
    (snapshot).  Yields (lo, hi, owner)."""
    b = piece_bounds(u_len, old_dp)
    out = []
    if alive[h]:
        out.append((b[h], b[h + 1], h))
        nxt = (h + 1) % old_dp
        if not alive[nxt] and nxt != h:
            out.append((b[nxt], b[nxt + 1], nxt))
    out.sort()
    return out


def staging(old_shards, snapshots, old_dp, new_dp, alive_mask, starts):
    """Contents of the staging arena: for every pair (holder h, new rank k)
    with new_rank(h) != k, the elements h serves that k will own, units in
    ascending order, ascending element order inside a unit.  Messages are laid
    out sorted by (k, h).  Returns (arena, {(h, k): (offset, length)})."""
    alive = alive_list(old_dp, alive_mask)
    flat = reconstruct_flat(old_shards, snapshots, old_dp, alive, starts)
    nro = new_rank_of(old_dp, new_dp, alive)
    msgs, table, off = [], {}, 0
    for k in range(new_dp):
        for h in range(old_dp):
            if not alive[h] or nro[h] == k:
                continue
            parts = []
            for u in range(len(starts) - 1):
                s = int(starts[u])
                L = int(starts[u + 1]) - s
                nb = piece_bounds(L, new_dp)
                for lo, hi, _owner in held_ranges(L, h, old_dp, alive):
                    a, z = max(lo, nb[k]), min(hi, nb[k + 1])
                    if a < z:
                        parts.append(flat[s + a:s + z])
            n = sum(len(p) for p in parts)
            if n:
                table[(h, k)] = (off, n)
                msgs.extend(parts)
                off += n
    arena = np.concatenate(msgs) if msgs else flat[:0].copy()
    return arena, table


# --------------------------------------------------------------------------
# one-by-one element map for sampled checks at any size (vectorised index
# arithmetic; pinned against brute.py on tiny inputs)
# --------------------------------------------------------------------------
def _bounds_matrix(starts: np.ndarray, D: int) -> np.ndarray:
    L = np.diff(np.asarray(starts, dtype=np.int64))
    n_gran = -(-L // GRANULE)
    j = np.arange(D + 1, dtype=np.int64)[None, :]
    return np.minimum(L[:, None], GRANULE * ((j * n_gran[:, None]) // D))


def locate_new_elements(starts, old_dp, new_dp, new_rank: int, offsets):
    """For positions `offsets` inside new shard `new_rank` return
    (global index, old owner, offset inside the old owner's shard)."""
    starts = np.asarray(starts, dtype=np.int64)
    offsets = np.asarray(offsets, dtype=np.int64)
    nb = _bounds_matrix(starts, new_dp)
    ob = _bounds_matrix(starts, old_dp)
    n_len = nb[:, new_rank + 1] - nb[:, new_rank]
    n_cum = np.concatenate([[0], np.cumsum(n_len)])
    u = np.searchsorted(n_cum, offsets, side="right") - 1
    p = nb[u, new_rank] + (offsets - n_cum[u])            # position inside the unit
    glob = starts[u] + p
    # old owner: last j with b_j <= p among non-empty pieces
    owner = (ob[u, 1:] <= p[:, None]).sum(axis=1)
    o_len = ob[:, 1:] - ob[:, :-1]
    o_cum = np.concatenate([np.zeros((1, old_dp), np.int64), np.cumsum(o_len, axis=0)])
    old_off = o_cum[u, owner] + (p - ob[u, owner])
    return glob, owner, old_off
