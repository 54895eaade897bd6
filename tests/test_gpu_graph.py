"""The launch-bound case: at the Tiny workload a step is ~40 kernel launches of a few microseconds
each, so the calls are captured once into a HIP graph and replayed.  Every replay is checked against
the eager result on fresh inputs (the library zero-fills with kernels, never with memset nodes)."""
import numpy as np
import pytest
import torch

import paper_2510_00606_amd as ew
from paper_2510_00606_amd import configs, synth

from gpu_util import DEV

pytestmark = pytest.mark.gpu


def test_step_replays_from_a_hip_graph():
    w = configs.tiny()
    A, es = synth.ARRAYS, synth.ELEM_SIZE
    plan = ew.ew_plan(w.old_dp, w.new_dp, w.alive_mask, w.numel, w.chunk)
    side = torch.cuda.Stream()
    ew.ew_plan_upload(plan, 0, side.cuda_stream)
    side.synchronize()
    old_len = [plan.old_shard_len(j) for j in range(w.old_dp)]
    new_len = [plan.new_shard_len(k) for k in range(w.new_dp)]
    alive = [(w.alive_mask >> j) & 1 for j in range(w.old_dp)]

    def buffers():
        b = {"old": {a: [torch.zeros(n, dtype=synth.TORCH_DTYPE[a], device=DEV) for n in old_len] for a in A}}
        b["snap"] = {a: [torch.zeros_like(t) for t in b["old"][a]] for a in A}
        b["sums"] = {a: [torch.zeros((ew.num_blocks(n * es[a]), 2), dtype=torch.int64, device=DEV) for n in old_len] for a in A}
        b["stage"] = {a: torch.zeros(plan.stage_len, dtype=synth.TORCH_DTYPE[a], device=DEV) for a in A}
        b["new"] = {a: [torch.zeros(n, dtype=synth.TORCH_DTYPE[a], device=DEV) for n in new_len] for a in A}
        b["nsnap"] = {a: [torch.zeros_like(t) for t in b["new"][a]] for a in A}
        b["nsums"] = {a: [torch.zeros((ew.num_blocks(n * es[a]), 2), dtype=torch.int64, device=DEV) for n in new_len] for a in A}
        return b

    def enqueue(b, st):
        for a in A:
            for j in range(w.old_dp):
                ew.ew_snapshot(b["old"][a][j], b["snap"][a][j], old_len[j] * es[a], b["sums"][a][j], st)
        for a in A:
            live = [t if alive[j] else None for j, t in enumerate(b["old"][a])]
            snaps = [None if alive[j] else t for j, t in enumerate(b["snap"][a])]
            ew.ew_pack(plan, live, snaps, b["stage"][a], es[a], st)
            ew.ew_unpack_snapshot(plan, b["stage"][a], live, snaps, b["new"][a], b["nsnap"][a], b["nsums"][a], es[a], st)

    def fill(b, seed):
        for a in A:
            for j in range(w.old_dp):
                b["old"][a][j].copy_(synth.fill(seed, j, a, 0, old_len[j], DEV))

    g_buf, e_buf = buffers(), buffers()
    # warm-up on the capture stream (first use of a stream claims its scratch region), then capture
    with torch.cuda.stream(side):
        enqueue(g_buf, side.cuda_stream)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        enqueue(g_buf, torch.cuda.current_stream().cuda_stream)
    for rep, seed in enumerate((11, 12, 13, 14)):
        fill(g_buf, seed)
        fill(e_buf, seed)
        torch.cuda.synchronize()
        graph.replay()
        enqueue(e_buf, torch.cuda.current_stream().cuda_stream)   # eager, default stream
        torch.cuda.synchronize()
        for key in ("snap", "sums", "new", "nsnap", "nsums"):
            for a in A:
                for x, y in zip(g_buf[key][a], e_buf[key][a]):
                    assert torch.equal(x.view(torch.uint8), y.view(torch.uint8)), f"replay {rep}: {key}/{a} differs"
        # and the eager result is not trivially zero
        assert int(e_buf["nsums"]["W"][0][:, 0].abs().sum().item()) != 0
    plan.close()
