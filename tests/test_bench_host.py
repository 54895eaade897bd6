"""Host-side checks of bench.py's own arithmetic (no GPU): the byte count of the CPU-baseline leg comes
from the oracle's layout functions alone and must agree with the planner's arena length on every
workload; the baseline leg itself runs on the tiny workload, on one thread and on several."""
import numpy as np

import bench
import paper_2510_00606_amd as ew
from oracle import layout
from paper_2510_00606_amd import configs, synth


def test_oracle_side_arena_length_equals_the_planners():
    for name in ("tiny", "7b_stage", "13b_stage", "70b_stage"):
        w = configs.ALL[name]()
        starts = w.unit_starts()
        with ew.ew_plan_bounds(w.old_dp, w.new_dp, w.alive_mask, starts) as p:
            want = p.stage_len
        got = bench.oracle_remote_elems(layout, starts.astype(np.int64), w.old_dp, w.new_dp, w.alive_mask)
        assert got == want, name
    # a ragged case with two failures
    starts = np.array([0, 1000, 1000, 5096, 5103, 9000], dtype=np.int64)
    with ew.ew_plan_bounds(6, 4, 0b101011, starts.astype(np.uint64)) as p:
        assert bench.oracle_remote_elems(layout, starts, 6, 4, 0b101011) == p.stage_len


def test_cpu_baseline_leg_runs_without_the_library():
    w = configs.tiny()
    starts = w.unit_starts()
    lens = layout.shard_lengths(starts.astype(np.int64), w.old_dp)
    host = {a: [synth.to_numpy_bits(synth.fill(w.seed, j, a, 0, lens[j], "cpu")) for j in range(w.old_dp)]
            for a in synth.ARRAYS}
    one = bench.cpu_baseline(w, starts, host, len(starts) - 1, 1)
    four = bench.cpu_baseline(w, starts, host, len(starts) - 1, 4)
    assert one[0] == four[0] > 0 and one[1] > 0 and four[1] > 0
    # bytes: snapshot of every old partition (2 x 14 B), verify of the failed one, snapshot of the new
    # partitions (2 x 14 B), pack + unpack under the unfused accounting (28 B x (N + remote))
    n, rem = w.numel, bench.oracle_remote_elems(layout, starts.astype(np.int64), w.old_dp, w.new_dp, w.alive_mask)
    assert one[0] == 28 * n + 14 * lens[2] + 28 * n + 28 * (n + rem)
