"""Layer migration between two pipeline stages of equal DP degree (CPU oracle).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Sec. 6.3 compares two ZeRO assignments when the optimizer state O_i of a layer
moves from stage S to stage S+1:

  contiguous   each DP group keeps ONE flat array of its stage's state and rank r
               owns one contiguous block of (about) 1/D of it; taking a layer out
               of (or putting one into) the array shifts every cut point, so data
               must be re-compacted inside both groups (Fig. 10a);
  interleaved  every layer is split uniformly and rank j owns piece j of every
               layer; rank j of stage S just hands its piece to rank j of stage
               S+1 (Fig. 10b).

The result is defined, as for a DP-degree change, by reconstruct -> re-slice:
gather both stages' flat arrays from the old shards, move the last `n_move`
units (layers) of stage S to the front of stage S+1, and slice the two new flat
arrays with the same assignment rule.  "Uniformly" / "approximately equal" with a
remainder is read as the granule floor split of layout.piece_bounds in both rules
(contiguous = one such split of the whole stage array).

Global rank numbering used for traffic statistics: stage S ranks are 0..D-1,
stage S+1 ranks are D..2D-1.
"""
from __future__ import annotations

import numpy as np

from .layout import piece_bounds

INTERLEAVED, CONTIGUOUS = 0, 1


def rank_intervals(starts, D: int, assignment: int):
    """For each rank the (lo, hi) element intervals of the stage's flat array it owns, in
    shard order."""
    starts = [int(x) for x in starts]
    out = [[] for _ in range(D)]
    if assignment == CONTIGUOUS:
        b = piece_bounds(starts[-1], D)
        for j in range(D):
            if b[j + 1] > b[j]:
                out[j].append((b[j], b[j + 1]))
        return out
    for u in range(len(starts) - 1):
        b = piece_bounds(starts[u + 1] - starts[u], D)
        for j in range(D):
            if b[j + 1] > b[j]:
                out[j].append((starts[u] + b[j], starts[u] + b[j + 1]))
    return out


def gather(shards, starts, D: int, assignment: int) -> np.ndarray:
    flat = np.empty(int(starts[-1]), dtype=np.asarray(shards[0]).dtype)
    for j, iv in enumerate(rank_intervals(starts, D, assignment)):
        cur = 0
        for lo, hi in iv:
            flat[lo:hi] = shards[j][cur:cur + hi - lo]
            cur += hi - lo
        if cur != len(shards[j]):
            raise ValueError(f"shard {j} has {len(shards[j])} elements, the assignment says {cur}")
    return flat


def scatter(flat, starts, D: int, assignment: int):
    out = []
    for iv in rank_intervals(starts, D, assignment):
        parts = [flat[lo:hi] for lo, hi in iv]
        out.append(np.concatenate(parts) if parts else flat[:0].copy())
    return out


def moved_starts(src_starts, dst_starts, n_move: int):
    """Unit boundaries of the two stages after the last n_move units of stage S have become
    the first units of stage S+1."""
    src = [int(x) for x in src_starts]
    dst = [int(x) for x in dst_starts]
    a = len(src) - 1
    if not 0 <= n_move <= a:
        raise ValueError("n_move out of range")
    cut = src[a - n_move]
    new_src = src[:a - n_move + 1]
    moved = [x - cut for x in src[a - n_move:]]          # 0 .. moved length
    new_dst = moved + [moved[-1] + x for x in dst[1:]]
    return np.asarray(new_src, np.int64), np.asarray(new_dst, np.int64), cut


def migrate(src_shards, dst_shards, src_starts, dst_starts, D: int, assignment: int, n_move: int):
    """New shards of stage S and stage S+1 after the migration."""
    flat_s = gather(src_shards, src_starts, D, assignment)
    flat_d = gather(dst_shards, dst_starts, D, assignment)
    new_src, new_dst, cut = moved_starts(src_starts, dst_starts, n_move)
    new_flat_s = flat_s[:cut]
    new_flat_d = np.concatenate([flat_s[cut:], flat_d])
    return scatter(new_flat_s, new_src, D, assignment), scatter(new_flat_d, new_dst, D, assignment)


def owner_map(starts, D: int, assignment: int, rank_base: int) -> np.ndarray:
    """Global rank owning each element of a stage's flat array."""
    own = np.empty(int(starts[-1]), dtype=np.int64)
    for j, iv in enumerate(rank_intervals(starts, D, assignment)):
        for lo, hi in iv:
            own[lo:hi] = rank_base + j
    return own


def traffic(src_starts, dst_starts, D: int, assignment: int, n_move: int):
    """Elements that change owner, as a (2D x 2D) matrix [old global rank, new global rank]
    with the diagonal (data that stays) included."""
    new_src, new_dst, cut = moved_starts(src_starts, dst_starts, n_move)
    old = np.concatenate([owner_map(src_starts, D, assignment, 0), owner_map(dst_starts, D, assignment, D)])
    new = np.concatenate([owner_map(new_src, D, assignment, 0), owner_map(new_dst, D, assignment, D)])
    m = np.zeros((2 * D, 2 * D), dtype=np.int64)
    np.add.at(m, (old, new), 1)
    return m


def split_traffic(m: np.ndarray, D: int):
    """(intra stage S, cross stage, intra stage S+1) elements that change owner."""
    off = m - np.diag(np.diag(m))
    return int(off[:D, :D].sum()), int(off[:D, D:].sum() + off[D:, :D].sum()), int(off[D:, D:].sum())
