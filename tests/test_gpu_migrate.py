"""GPU parity of layer-migration plans (Sec. 6.3): ew_plan_migrate executed by ew_pack / ew_unpack /
ew_unpack_snapshot and by the arena-free ew_reshard against oracle/migrate.py, both ZeRO assignments,
bit for bit."""
import numpy as np
import pytest
import torch

import paper_2510_00606_amd as ew
from oracle import checksum, migrate
from paper_2510_00606_amd import configs, synth

from gpu_util import DEV, guard_intact, guarded, np_bits, stream, to_dev

pytestmark = pytest.mark.gpu


def run_case(assignment, D, src, dst, n_move, elem_size, rng):
    src, dst = np.asarray(src, np.int64), np.asarray(dst, np.int64)
    npdt = {2: np.uint16, 4: np.uint32}[elem_size]
    lens = [sum(h - l for l, h in x) for x in migrate.rank_intervals(src, D, assignment)] + \
           [sum(h - l for l, h in x) for x in migrate.rank_intervals(dst, D, assignment)]
    host = [rng.integers(0, 1 << (8 * elem_size), n, dtype=np.uint64).astype(npdt) for n in lens]
    want_s, want_d = migrate.migrate(host[:D], host[D:], src, dst, D, assignment, n_move)
    want = want_s + want_d
    plan = ew.ew_plan_migrate(assignment, D, src, dst, n_move)
    ew.ew_plan_upload(plan, 0, stream())
    old = [to_dev(h, elem_size) for h in host]
    stage = guarded(plan.stage_len, elem_size)
    new = [guarded(plan.new_shard_len(k), elem_size) for k in range(2 * D)]
    ew.ew_pack(plan, old, None, stage, elem_size, stream())
    ew.ew_unpack(plan, stage, old, None, new, elem_size, stream())
    new2 = [guarded(plan.new_shard_len(k), elem_size) for k in range(2 * D)]
    snap2 = [guarded(plan.new_shard_len(k), elem_size) for k in range(2 * D)]
    ck2 = [torch.zeros((ew.num_blocks(plan.new_shard_len(k) * elem_size), 2), dtype=torch.int64, device=DEV)
           for k in range(2 * D)]
    ew.ew_unpack_snapshot(plan, stage, old, None, new2, snap2, ck2, elem_size, stream())
    new3 = [guarded(plan.new_shard_len(k), elem_size) for k in range(2 * D)]
    ew.ew_reshard(plan, old, None, new3, elem_size, stream())   # no arena: rank j of stage S+1 pulls from rank j of stage S
    torch.cuda.synchronize()
    m = migrate.traffic(src, dst, D, assignment, n_move)
    assert plan.stage_len == int(m.sum() - np.trace(m))
    assert guard_intact(stage, plan.stage_len, elem_size)
    for k in range(2 * D):
        n = plan.new_shard_len(k)
        assert n == len(want[k])
        for got in (new[k], new2[k], snap2[k], new3[k]):
            assert np.array_equal(np_bits(got[:n]), want[k]), f"rank {k} differs"
            assert guard_intact(got, n, elem_size)
        assert np.array_equal(ck2[k].cpu().numpy().view(np.uint64), checksum.block_checksums(want[k]))
    plan.close()


@pytest.mark.parametrize("assignment", [ew.EW_ASSIGN_INTERLEAVED, ew.EW_ASSIGN_CONTIGUOUS])
@pytest.mark.parametrize("elem_size", [2, 4])
def test_migrate_small_and_ragged(assignment, elem_size):
    rng = np.random.default_rng(assignment * 10 + elem_size)
    for D, src, dst, n_move in [(3, [0, 100, 364, 1000], [0, 264, 500], 2), (4, [0, 8, 16, 4099], [0, 7], 1),
                                (2, [0, 50, 120], [0, 30, 90, 91], 0), (5, [0, 1000], [0, 24, 48], 1),
                                (4, list(range(0, 400001, 25000)), list(range(0, 200001, 25000)), 5),
                                (8, list(range(0, 64 * 6401, 6400)), list(range(0, 64 * 3201, 6400)), 7),
                                (32, [0, 500000, 1000000], [0, 500000], 1)]:
        run_case(assignment, D, src, dst, n_move, elem_size, rng)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("assignment", [ew.EW_ASSIGN_INTERLEAVED, ew.EW_ASSIGN_CONTIGUOUS])
def test_migrate_one_llama_layer(assignment):
    """Two stages of two Llama-7B-shaped layers each, DP 8, one layer moves; units of 262 144 elements
    cut at tensor starts; bf16 and fp32, everything compared with the oracle."""
    w = configs.Workload("migrate", 9, configs.stage_tensors(4096, 11008, 2), 8, 8, 0xFF, 262144, snap_to_tensors=True)
    starts = w.unit_starts().astype(np.int64)
    per_layer = (len(starts) - 1) // 2
    rng = np.random.default_rng(assignment)
    for es in (2, 4):
        run_case(assignment, 8, starts, starts, per_layer, es, rng)
