"""Per-block checksums of a byte buffer and their verification (CPU oracle).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The abstract names verification of the snapshots while training runs, and the
paper never defines the check.  Definition used here: the buffer's bytes are read as
little-endian 64-bit words (a trailing partial word is zero-padded); block b
covers bytes [b*2^20, min((b+1)*2^20, nbytes)); its record is
(sum of its words mod 2^64, XOR of its words).  Both are order-independent,
so any reduction tree gives the same bits.
"""
from __future__ import annotations

import numpy as np

BLOCK_BYTES = 1 << 20
WORDS_PER_BLOCK = BLOCK_BYTES // 8


def as_words(buf) -> np.ndarray:
    raw = np.ascontiguousarray(buf).view(np.uint8).reshape(-1)
    pad = (-len(raw)) % 8
    if pad:
        raw = np.concatenate([raw, np.zeros(pad, np.uint8)])
    return raw.view("<u8")


def block_checksums(buf) -> np.ndarray:
    """(n_blocks, 2) uint64: column 0 = wrapping sum, column 1 = XOR."""
    w = as_words(buf)
    nbytes = np.ascontiguousarray(buf).nbytes
    n_blocks = -(-nbytes // BLOCK_BYTES)
    out = np.zeros((n_blocks, 2), dtype=np.uint64)
    for b in range(n_blocks):
        blk = w[b * WORDS_PER_BLOCK:(b + 1) * WORDS_PER_BLOCK]
        out[b, 0] = np.add.reduce(blk, dtype=np.uint64)
        out[b, 1] = np.bitwise_xor.reduce(blk)
    return out


def verify(buf, stored: np.ndarray):
    """Blocks whose recomputed record differs from `stored`, ascending, with
    (sum_now - sum_stored mod 2^64, xor_now ^ xor_stored) for each."""
    now = block_checksums(buf)
    stored = np.asarray(stored, dtype=np.uint64).reshape(-1, 2)
    if now.shape != stored.shape:
        raise ValueError("checksum array has the wrong number of blocks")
    bad = np.nonzero((now != stored).any(axis=1))[0]
    diffs = np.stack([now[bad, 0] - stored[bad, 0], now[bad, 1] ^ stored[bad, 1]], axis=1)
    return bad.astype(np.int64), diffs
