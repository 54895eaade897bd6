"""The five workloads (shapes, DP change, failed ranks, interleave units) used by the tests and
bench.py.  Shapes only: the state's values come from synth.py.  The tensor lists follow the
public Llama architecture descriptions (per layer: input norm, q, k, v, o projections, post-
attention norm, gate, up, down projections); they stand in for the paper's Llama-2 training
jobs (Table 2), whose weights are neither available nor needed by a path that moves bytes.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 0x25100606


def llama_layer_tensors(d: int, ffn: int, kv: int | None = None) -> list[int]:
    kv = d if kv is None else kv
    return [d, d * d, d * kv, d * kv, d * d, d, ffn * d, ffn * d, d * ffn]


def stage_tensors(d: int, ffn: int, layers: int, kv: int | None = None, vocab: int = 0) -> list[int]:
    t = [vocab * d] if vocab else []
    for _ in range(layers):
        t += llama_layer_tensors(d, ffn, kv)
    return t


@dataclass
class Workload:
    name: str
    index: int
    tensors: list[int]
    old_dp: int
    new_dp: int
    alive_mask: int
    chunk: int                      # nominal interleave chunk, elements
    snap_to_tensors: bool = False   # unit boundaries also at every tensor start
    note: str = ""
    seed: int = field(init=False)

    def __post_init__(self):
        self.seed = BASE_SEED + self.index

    @property
    def numel(self) -> int:
        return int(sum(self.tensors))

    @property
    def failed(self) -> list[int]:
        return [j for j in range(self.old_dp) if not (self.alive_mask >> j) & 1]

    def unit_starts(self) -> np.ndarray:
        """Boundaries of the interleave units (the paper's layers), n_units + 1 values."""
        n, c = self.numel, self.chunk
        if not self.snap_to_tensors:
            return np.asarray(list(range(0, n, c)) + [n], dtype=np.uint64)
        cuts, base = [], 0
        for t in self.tensors:
            cuts.extend(range(base, base + t, c))
            base += t
        cuts.append(n)
        return np.asarray(cuts, dtype=np.uint64)


def _seeded_failures(seed: int, old_dp: int, n_fail: int) -> int:
    """n_fail distinct failed ranks, redrawn until none of them is the ring predecessor of
    another (otherwise a snapshot and its owner are lost together)."""
    rng = np.random.default_rng([seed, 99])
    while True:
        f = sorted(int(x) for x in rng.choice(old_dp, size=n_fail, replace=False))
        if all(((x - 1) % old_dp) not in f for x in f):
            mask = (1 << old_dp) - 1
            for x in f:
                mask &= ~(1 << x)
            return mask


def tiny() -> Workload:
    return Workload("tiny", 0, [1 << 20], 4, 3, 0b1011, 4096, note="DP 4->3, rank 2 failed")


def stage_7b() -> Workload:
    return Workload("7b_stage", 1, stage_tensors(4096, 11008, 8, vocab=32000), 8, 7, 0xFF & ~(1 << 5), 262144,
                    note="Llama-7B shape: embedding + 8 of 32 layers, DP 8->7, rank 5 failed")


def snapshot_7b() -> Workload:
    # one rank's shard of the 7B stage: every unit of the stage splits evenly over 8 ranks
    w = stage_7b()
    return Workload("7b_rank_snapshot", 2, [w.numel // 8], 1, 1, 1, w.numel // 8,
                    note="old rank 0's shard of the 7B stage: snapshot + checksum + bit-flip search")


def stage_13b() -> Workload:
    w = Workload("13b_stage", 3, stage_tensors(5120, 13824, 10), 16, 12, 0, 262144, snap_to_tensors=True,
                 note="Llama-13B shape: 10 of 40 layers, DP 16->12, 4 seeded failures, units cut at tensor starts")
    w.alive_mask = _seeded_failures(w.seed, 16, 4)
    return w


def stage_70b() -> Workload:
    return Workload("70b_stage", 4, stage_tensors(8192, 28672, 10, kv=1024), 7, 8, 0x7F, 1 << 20,
                    note="Llama-70B shape (GQA, 8 KV heads): 10 of 80 layers, DP 7->8, one rank joins")


ALL = {"tiny": tiny, "7b_stage": stage_7b, "7b_rank_snapshot": snapshot_7b, "13b_stage": stage_13b,
       "70b_stage": stage_70b}
