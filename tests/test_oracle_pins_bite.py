"""Do the pins bite?  Each case plants ONE plausible mistake in the CPU oracle (a dropped term, a
wrong sign or index, a swapped order) and runs that oracle's pins: at least one of them must fail.
The mistakes live on the CPU only and are undone after each case.  A mistake that no pin notices
would mean the oracle is free to be wrong in that way, and with it every parity claim.  (That the
unmodified oracle passes every pin is what the pins' own test modules check.)
"""
import numpy as np
import pytest

import test_oracle_adam as TA
import test_oracle_checksum as TC
import test_oracle_layout as TL
import test_oracle_migrate as TM
import test_partition as TP
from oracle import adam, checksum, layout, migrate, partition

LAYOUT_PINS = [
    TL.test_paper_scenario_d4_f2, TL.test_snapshot_holder_is_ring_predecessor, TL.test_piece_bounds_properties,
    TL.test_every_rank_owns_a_piece_of_every_unit, lambda: TL.test_scale_up_local_fraction_is_half(3),
    lambda: TL.test_scale_up_local_fraction_is_half(4), TL.test_identity_when_nothing_changes,
    TL.test_single_unit_is_numpy_split, TL.test_gather_and_scatter_extremes, TL.test_round_trip_restores_old_shards,
    TL.test_brute_force_larger_ragged, TL.test_failed_live_shards_are_never_read,
]
CHECKSUM_PINS = [
    TC.test_zero_block, TC.test_all_ones_words, TC.test_ramp_words, TC.test_wraparound,
    lambda: TC.test_against_bigint(17), lambda: TC.test_against_bigint((1 << 20) + 1), TC.test_little_endian_word_order,
    TC.test_dtype_views_agree, lambda: TC.test_single_bit_flip_algebra(0), TC.test_verify_lists_blocks_ascending,
]
MIGRATE_PINS = [
    lambda: TM.test_interleaved_is_D_one_to_one_sends(4), lambda: TM.test_contiguous_closed_form(4),
    TM.test_contiguous_stage_is_numpy_split, TM.test_interleaved_stage_matches_layout_module,
    lambda: TM.test_migration_preserves_the_logical_state(migrate.INTERLEAVED),
    lambda: TM.test_migration_preserves_the_logical_state(migrate.CONTIGUOUS),
    TM.test_interleaved_rank_keeps_piece_j_of_every_layer, TM.test_hand_worked_migration_of_unequal_layers,
]
ADAM_PINS = [
    TA.test_first_step_closed_form, TA.test_zero_gradient_decays_moments_and_applies_weight_decay_only,
    TA.test_against_float64_and_torch_adamw, TA.test_bf16_gradient_widens_exactly, TA.test_hyper_scalars,
    TA.test_bf16_rounding_by_hand, TA.test_bf16_rounding_matches_integer_rule_on_random_bits,
]
# the pins of the bf16 rounding that call no conversion routine of any library
BF16_PINS = [TA.test_bf16_rounding_by_hand, TA.test_bf16_rounding_matches_integer_rule_on_random_bits]
PARTITION_PINS = [TP.test_oracle_closed_forms]   # the one that involves the oracle alone


def failures(pins):
    n = 0
    for pin in pins:
        try:
            pin()
        except Exception:  # an assertion, or the mistake trips a consistency check inside the oracle
            n += 1
    return n


# ------------------------------------------------------------------ layout.py
def _bounds_floor_granules(L, D):      # granule count rounded down: the ragged tail is lost to the last cut
    n = L // layout.GRANULE
    return [0] + [min(L, layout.GRANULE * ((j * n) // D)) for j in range(1, D)] + [L]


def _bounds_ceil_split(L, D):          # cuts rounded up instead of down
    n = -(-L // layout.GRANULE)
    return [min(L, layout.GRANULE * (-(-(j * n) // D))) for j in range(D + 1)]


def _bounds_no_granule(L, D):          # element-exact split, no 8-element granule
    return [(j * L) // D for j in range(D + 1)]


def _holder_successor(owner, old_dp, alive):   # snapshot looked for at the ring successor
    if alive[owner]:
        return owner
    h = (owner + 1) % old_dp
    if not alive[h]:
        raise layout.Unrecoverable("both failed")
    return h


def _new_rank_reversed(old_dp, new_dp, alive):  # survivors renumbered from the top
    out, nxt = [-1] * old_dp, 0
    for j in reversed(range(old_dp)):
        if alive[j] and nxt < new_dp:
            out[j] = nxt
            nxt += 1
    return out


def _reconstruct_reads_dead_devices(old_shards, snapshots, old_dp, alive, starts, _orig=layout.reconstruct_flat):
    return _orig(old_shards, [None] * old_dp, old_dp, [True] * old_dp, starts)   # never consults a snapshot


def _slice_rank_major(flat, new_dp, starts):   # contiguous split of the whole array instead of unit by unit
    return [np.array(x) for x in np.array_split(np.asarray(flat), new_dp)]


def _held_ranges_own_piece_only(u_len, h, old_dp, alive):   # forgets the failed successor's piece
    b = layout.piece_bounds(u_len, old_dp)
    return [(b[h], b[h + 1], h)] if alive[h] else []


LAYOUT_MISTAKES = {
    "granule count rounded down": ("piece_bounds", _bounds_floor_granules),
    "cuts rounded up": ("piece_bounds", _bounds_ceil_split),
    "no granule": ("piece_bounds", _bounds_no_granule),
    "snapshot at ring successor": ("holder_of", _holder_successor),
    "survivors renumbered from the top": ("new_rank_of", _new_rank_reversed),
    "failed ranks' devices are read": ("reconstruct_flat", _reconstruct_reads_dead_devices),
    "contiguous instead of interleaved slicing": ("slice_flat", _slice_rank_major),
    "holder serves only its own piece": ("held_ranges", _held_ranges_own_piece_only),
}


@pytest.mark.parametrize("name", sorted(LAYOUT_MISTAKES))
def test_layout_pins_catch(name, monkeypatch):
    attr, wrong = LAYOUT_MISTAKES[name]
    monkeypatch.setattr(layout, attr, wrong)
    assert failures(LAYOUT_PINS) > 0, f"no layout pin notices: {name}"


# ------------------------------------------------------------------ checksum.py
def _words_big_endian(buf):
    raw = np.ascontiguousarray(buf).view(np.uint8).reshape(-1)
    raw = np.concatenate([raw, np.zeros((-len(raw)) % 8, np.uint8)])
    return raw.view(">u8").astype(np.uint64)


def _words_tail_padded_with_ones(buf):
    raw = np.ascontiguousarray(buf).view(np.uint8).reshape(-1)
    raw = np.concatenate([raw, np.full((-len(raw)) % 8, 0xFF, np.uint8)])
    return raw.view("<u8")


def _blocks(buf, words_per_block=checksum.WORDS_PER_BLOCK, sum_of=lambda blk: np.add.reduce(blk, dtype=np.uint64),
            xor_of=np.bitwise_xor.reduce):
    w = checksum.as_words(buf)
    nbytes = np.ascontiguousarray(buf).nbytes
    n_blocks = -(-nbytes // (8 * words_per_block))
    out = np.zeros((n_blocks, 2), dtype=np.uint64)
    for b in range(n_blocks):
        blk = w[b * words_per_block:(b + 1) * words_per_block]
        out[b, 0] = sum_of(blk)
        out[b, 1] = xor_of(blk)
    return out


def _verify_unsorted(buf, stored, _orig=checksum.verify):
    bad, diffs = _orig(buf, stored)
    return bad[::-1], diffs[::-1]


def _verify_wrong_sign(buf, stored, _orig=checksum.verify):
    bad, diffs = _orig(buf, stored)
    diffs = diffs.copy()
    diffs[:, 0] = np.uint64(0) - diffs[:, 0]
    return bad, diffs


CHECKSUM_MISTAKES = {
    "big-endian words": ("as_words", _words_big_endian),
    "tail padded with ones": ("as_words", _words_tail_padded_with_ones),
    "block of 2^20 words": ("block_checksums", lambda buf: _blocks(buf, words_per_block=1 << 20)),
    "sum saturates instead of wrapping": ("block_checksums", lambda buf: _blocks(
        buf, sum_of=lambda blk: np.uint64(min(sum(int(x) for x in blk[:4096]) + int(np.add.reduce(blk[4096:], dtype=np.uint64)),
                                               (1 << 64) - 1)))),
    "or instead of xor": ("block_checksums", lambda buf: _blocks(buf, xor_of=np.bitwise_or.reduce)),
    "bad blocks listed descending": ("verify", _verify_unsorted),
    "sum difference with the wrong sign": ("verify", _verify_wrong_sign),
}


@pytest.mark.parametrize("name", sorted(CHECKSUM_MISTAKES))
def test_checksum_pins_catch(name, monkeypatch):
    attr, wrong = CHECKSUM_MISTAKES[name]
    monkeypatch.setattr(checksum, attr, wrong)
    assert failures(CHECKSUM_PINS) > 0, f"no checksum pin notices: {name}"


# ------------------------------------------------------------------ adam.py
def _adam_variant(**change):
    F = np.float32

    def step(w, m, v, g, h):
        g = adam.grad_to_f32(g)
        with np.errstate(all="ignore"):
            m = F(h["beta1"]) * m + F(h["omb1"]) * g
            v = F(h["beta2"]) * v + F(h["omb2"]) * (g if change.get("v_not_squared") else g * g)
            vhat = v if change.get("no_bias2") else v * F(h["bias2"])
            den = np.sqrt(vhat) + F(h["eps"])
            mhat = m if change.get("no_bias1") else m * F(h["bias1"])
            upd = mhat / den
            decay = F(0) * w if change.get("no_decay") else F(h["wd"]) * w
            w = w + F(h["lr"]) * (upd + decay) if change.get("ascent") else w - F(h["lr"]) * (upd + decay)
        return w, m, v, adam.bf16_bits(w)
    return step


def _bf16_truncate(w):
    return (np.ascontiguousarray(w).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def _bf16_half_away(w):        # ties away from zero: add half a unit to the magnitude, then truncate
    u = np.ascontiguousarray(w).view(np.uint32).astype(np.uint64)
    return ((u + np.uint64(0x8000)) >> np.uint64(16)).astype(np.uint16)


def _bf16_half_up(w):          # ties toward +infinity: away from zero for positives, toward zero for negatives
    u = np.ascontiguousarray(w).view(np.uint32).astype(np.uint64)
    neg = (u >> np.uint64(31)) == 1
    return ((u + np.where(neg, np.uint64(0x7FFF), np.uint64(0x8000))) >> np.uint64(16)).astype(np.uint16)


def _bf16_half_odd(w):         # ties to the odd neighbour
    u = np.ascontiguousarray(w).view(np.uint32).astype(np.uint64)
    return ((u + np.uint64(0x8000) - ((u >> np.uint64(16)) & np.uint64(1))) >> np.uint64(16)).astype(np.uint16)


BF16_MISTAKES = {
    "bf16 by truncation": _bf16_truncate,
    "bf16 ties away from zero": _bf16_half_away,
    "bf16 ties toward plus infinity": _bf16_half_up,
    "bf16 ties to odd": _bf16_half_odd,
}


@pytest.mark.parametrize("name", sorted(BF16_MISTAKES))
def test_bf16_pins_catch_without_any_library_conversion(name, monkeypatch):
    monkeypatch.setattr(adam, "bf16_bits", BF16_MISTAKES[name])
    for pin in BF16_PINS:       # each of the two pins notices each mistake on its own
        assert failures([pin]) == 1, f"{pin.__name__} does not notice: {name}"


ADAM_MISTAKES = {
    "second moment from g instead of g*g": ("step", _adam_variant(v_not_squared=True)),
    "no bias correction of m": ("step", _adam_variant(no_bias1=True)),
    "no bias correction of v": ("step", _adam_variant(no_bias2=True)),
    "weight decay dropped": ("step", _adam_variant(no_decay=True)),
    "update added instead of subtracted": ("step", _adam_variant(ascent=True)),
    "bf16 by truncation": ("bf16_bits", _bf16_truncate),
}


@pytest.mark.parametrize("name", sorted(ADAM_MISTAKES))
def test_adam_pins_catch(name, monkeypatch):
    attr, wrong = ADAM_MISTAKES[name]
    monkeypatch.setattr(adam, attr, wrong)
    assert failures(ADAM_PINS) > 0, f"no Adam pin notices: {name}"


# ------------------------------------------------------------------ migrate.py
def _moved_starts_from_the_front(src_starts, dst_starts, n_move):   # the FIRST layers of stage S leave
    src = [int(x) for x in src_starts]
    dst = [int(x) for x in dst_starts]
    cut = src[n_move]
    new_src = [x - cut for x in src[n_move:]]
    moved = src[:n_move + 1]
    new_dst = moved + [moved[-1] + x for x in dst[1:]]
    return np.asarray(new_src, np.int64), np.asarray(new_dst, np.int64), src[-1] - cut


def _migrate_appends(src_shards, dst_shards, src_starts, dst_starts, D, assignment, n_move):
    # moved layers land BEHIND stage S+1's own layers instead of in front of them
    flat_s = migrate.gather(src_shards, src_starts, D, assignment)
    flat_d = migrate.gather(dst_shards, dst_starts, D, assignment)
    new_src, new_dst, cut = migrate.moved_starts(src_starts, dst_starts, n_move)
    return (migrate.scatter(flat_s[:cut], new_src, D, assignment),
            migrate.scatter(np.concatenate([flat_d, flat_s[cut:]]), new_dst, D, assignment))


def _intervals_ignore_assignment(starts, D, assignment, _orig=migrate.rank_intervals):
    return _orig(starts, D, migrate.INTERLEAVED)


def _owner_map_without_stage_base(starts, D, assignment, rank_base, _orig=migrate.owner_map):
    return _orig(starts, D, assignment, 0)


def _split_counts_what_stays(m, D):
    return int(m[:D, :D].sum()), int(m[:D, D:].sum() + m[D:, :D].sum()), int(m[D:, D:].sum())


MIGRATE_MISTAKES = {
    "first layers move instead of last": ("moved_starts", _moved_starts_from_the_front),
    "moved layers appended behind": ("migrate", _migrate_appends),
    "contiguous rule treated as interleaved": ("rank_intervals", _intervals_ignore_assignment),
    "stage S+1 ranks numbered like stage S": ("owner_map", _owner_map_without_stage_base),
    "data that stays counted as traffic": ("split_traffic", _split_counts_what_stays),
    "no granule in the split": ("piece_bounds", _bounds_no_granule),
}


@pytest.mark.parametrize("name", sorted(MIGRATE_MISTAKES))
def test_migrate_pins_catch(name, monkeypatch):
    attr, wrong = MIGRATE_MISTAKES[name]
    monkeypatch.setattr(migrate, attr, wrong)
    assert failures(MIGRATE_PINS) > 0, f"no migration pin notices: {name}"


# ------------------------------------------------------------------ partition.py
def _partition_variant(combine=max, respect_cap=True, better=lambda new, best: new < best, stage=lambda p: p):
    import itertools
    import math

    def best_partition(L, P, t, mem, cap):
        best, arg = None, None
        for cuts in itertools.combinations(range(1, L), P - 1):
            edges = (0,) + cuts + (L,)
            worst, ok = 0.0, True
            for p in range(P):
                a, b = edges[p], edges[p + 1] - 1
                if respect_cap and mem[a][b] > cap[p]:
                    ok = False
                    break
                worst = combine(worst, t[stage(p)][a][b])
            if ok and (best is None or better(worst, best)):
                best, arg = worst, list(cuts)
        return (math.inf, None) if best is None else (best, arg)
    return best_partition


PARTITION_MISTAKES = {
    "sum of stage times instead of the maximum": _partition_variant(combine=lambda a, b: a + b),
    "memory caps ignored": _partition_variant(respect_cap=False),
    "worst partition kept": _partition_variant(better=lambda new, best: new > best),
    "every stage timed as stage 0": _partition_variant(stage=lambda p: 0),
}


@pytest.mark.parametrize("name", sorted(PARTITION_MISTAKES))
def test_partition_pins_catch(name, monkeypatch):
    monkeypatch.setattr(partition, "best_partition", PARTITION_MISTAKES[name])
    assert failures(PARTITION_PINS) > 0, f"no partition pin notices: {name}"
