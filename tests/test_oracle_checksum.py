"""Pins for oracle/checksum.py (CPU only): closed forms, Python big-int
arithmetic, bit-flip algebra."""
import numpy as np
import pytest

from oracle import checksum

M64 = (1 << 64) - 1
WPB = 131072  # 64-bit words per 1 MiB block


def bigint_blocks(raw: bytes):
    """Block records with Python integers only (no numpy arithmetic)."""
    out = []
    for b0 in range(0, len(raw), 1 << 20):
        blk = raw[b0:b0 + (1 << 20)]
        blk += b"\0" * ((-len(blk)) % 8)
        s = x = 0
        for i in range(0, len(blk), 8):
            w = int.from_bytes(blk[i:i + 8], "little")
            s = (s + w) & M64
            x ^= w
        out.append((s, x))
    return out


def test_zero_block():
    c = checksum.block_checksums(np.zeros(1 << 20, np.uint8))
    assert c.shape == (1, 2) and c[0, 0] == 0 and c[0, 1] == 0


def test_all_ones_words():
    for n in (1, 2, 3, 1000, 1001, WPB):
        c = checksum.block_checksums(np.full(n, M64, np.uint64))
        assert int(c[0, 0]) == (-n) & M64
        assert int(c[0, 1]) == (0 if n % 2 == 0 else M64)


def test_ramp_words():
    w = np.arange(WPB, dtype=np.uint64)
    c = checksum.block_checksums(w)
    assert int(c[0, 0]) == WPB * (WPB - 1) // 2 == 8589869056
    assert int(c[0, 1]) == 0  # XOR of 0..2^17-1 vanishes


def test_wraparound():
    w = np.array([M64, 1, 1 << 63, 1 << 63], dtype=np.uint64)
    c = checksum.block_checksums(w)
    assert int(c[0, 0]) == 0 and int(c[0, 1]) == (M64 ^ 1)


@pytest.mark.parametrize("nbytes", [0, 1, 7, 8, 9, 15, 16, 17, (1 << 20) - 1, 1 << 20, (1 << 20) + 1,
                                    (1 << 20) + 8, 3 * (1 << 20) + 12345])
def test_against_bigint(nbytes):
    rng = np.random.default_rng(nbytes)
    raw = rng.integers(0, 256, nbytes, dtype=np.uint8)
    c = checksum.block_checksums(raw)
    ref = bigint_blocks(raw.tobytes())
    assert c.shape[0] == len(ref) == -(-nbytes // (1 << 20))
    for b, (s, x) in enumerate(ref):
        assert int(c[b, 0]) == s and int(c[b, 1]) == x


def test_little_endian_word_order():
    raw = np.arange(1, 9, dtype=np.uint8)  # bytes 01..08 -> word 0x0807060504030201
    c = checksum.block_checksums(raw)
    assert int(c[0, 0]) == 0x0807060504030201
    raw = np.array([0xAB], dtype=np.uint8)  # zero-padded tail
    assert int(checksum.block_checksums(raw)[0, 1]) == 0xAB


def test_dtype_views_agree():
    rng = np.random.default_rng(11)
    f = rng.standard_normal(300001).astype(np.float32)
    assert np.array_equal(checksum.block_checksums(f), checksum.block_checksums(f.view(np.uint8)))


@pytest.mark.parametrize("seed", range(6))
def test_single_bit_flip_algebra(seed):
    rng = np.random.default_rng(100 + seed)
    nbytes = 5 * (1 << 20) + 4096 + 3
    raw = rng.integers(0, 256, nbytes, dtype=np.uint8)
    stored = checksum.block_checksums(raw)
    bad, diffs = checksum.verify(raw, stored)
    assert len(bad) == 0
    o = int(rng.integers(0, nbytes))
    beta = int(rng.integers(0, 8))
    was_set = (int(raw[o]) >> beta) & 1
    raw[o] ^= np.uint8(1 << beta)
    bad, diffs = checksum.verify(raw, stored)
    assert bad.tolist() == [o >> 20]
    onehot = 1 << (8 * (o % 8) + beta)
    assert int(diffs[0, 1]) == onehot
    assert int(diffs[0, 0]) == ((-onehot) & M64 if was_set else onehot)


def test_verify_lists_blocks_ascending():
    rng = np.random.default_rng(9)
    raw = rng.integers(0, 256, 8 << 20, dtype=np.uint8)
    stored = checksum.block_checksums(raw)
    for blk in (6, 1, 3):
        raw[(blk << 20) + 17] ^= 0x10
    bad, _ = checksum.verify(raw, stored)
    assert bad.tolist() == [1, 3, 6]
