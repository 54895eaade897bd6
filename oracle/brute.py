"""Per-element brute force for tiny sizes (CPU oracle, pure Python loops).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Independent of layout.py's slicing: it never computes a piece boundary.  An
element's owner is found by scanning ranks for the one whose run of 8-element
granules contains the element's granule, and an element's offset inside its
owner's shard is the number of lower-indexed elements with the same owner (a
rank's shard holds its elements in ascending global order: Fig. 10b, pieces of
successive layers laid one after the other).
"""
from __future__ import annotations


def owner_in_unit(pos: int, L: int, D: int) -> int:
    """Rank owning position `pos` of a unit of L elements split over D ranks:
    granule q belongs to the rank j with floor(j*G/D) <= q < floor((j+1)*G/D)."""
    n_gran = (L + 7) // 8
    q = pos // 8
    for j in range(D):
        if (j * n_gran) // D <= q < ((j + 1) * n_gran) // D:
            return j
    raise AssertionError("granule not covered")


def element_map(starts, D: int):
    """For every global element e: (unit, owner, offset in owner's shard)."""
    starts = [int(s) for s in starts]
    numel = starts[-1]
    count = [0] * D
    out = []
    u = 0
    for e in range(numel):
        while e >= starts[u + 1]:
            u += 1
        j = owner_in_unit(e - starts[u], starts[u + 1] - starts[u], D)
        out.append((u, j, count[j]))
        count[j] += 1
    return out, count


def reshard_map(starts, old_dp: int, new_dp: int, alive):
    """List over global elements of
    (old owner, old offset, reads_snapshot, holder, new rank, new offset)."""
    old, _ = element_map(starts, old_dp)
    new, new_len = element_map(starts, new_dp)
    out = []
    for (_, j, oo), (_, k, no) in zip(old, new):
        if alive[j]:
            holder, snap = j, False
        else:
            holder, snap = (j - 1) % old_dp, True
            if not alive[holder]:
                raise RuntimeError("unrecoverable")
        out.append((j, oo, snap, holder, k, no))
    return out, new_len
