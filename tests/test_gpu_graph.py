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


def test_four_capturing_streams_leave_eager_calls_working():
    """Four streams of one device each capture a fused unpack + snapshot.  Three of the captures tie a
    scratch region to their graph; the fourth would take the last region outside graphs, so it records
    the scratch-free kernels instead.  An eager call on a fifth stream still gets a region, every
    replay equals the eager result, and ew_scratch_release gives the regions back afterwards."""
    Do, Dn, mask, N, C, es = 5, 4, 0b11011, 700_000, 40_000, 4
    plan = ew.ew_plan(Do, Dn, mask, N, C)
    ew.ew_plan_upload(plan, 0, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    alive = [(mask >> j) & 1 for j in range(Do)]
    old_len = [plan.old_shard_len(j) for j in range(Do)]

    def buffers(seed):
        old = [synth.fill(seed, j, "W", 0, old_len[j], DEV) for j in range(Do)]
        live = [t if alive[j] else None for j, t in enumerate(old)]
        snaps = [None if alive[j] else t for j, t in enumerate(old)]
        stage = torch.zeros(plan.stage_len, dtype=torch.float32, device=DEV)
        new = [torch.zeros(plan.new_shard_len(k), dtype=torch.float32, device=DEV) for k in range(Dn)]
        nsn = [torch.zeros_like(t) for t in new]
        ck = [torch.zeros((ew.num_blocks(t.numel() * es), 2), dtype=torch.int64, device=DEV) for t in new]
        return live, snaps, stage, new, nsn, ck

    def enqueue(b, st):
        live, snaps, stage, new, nsn, ck = b
        ew.ew_pack(plan, live, snaps, stage, es, st)
        ew.ew_unpack_snapshot(plan, stage, live, snaps, new, nsn, ck, es, st)
        ew.ew_snapshot(new[0], nsn[0], new[0].numel() * es, ck[0], st)

    streams = [torch.cuda.Stream() for _ in range(4)]
    bufs = [buffers(40 + i) for i in range(4)]
    for s, b in zip(streams, bufs):           # warm-up: every stream claims a region
        with torch.cuda.stream(s):
            enqueue(b, s.cuda_stream)
    torch.cuda.synchronize()
    graphs = []
    for s, b in zip(streams, bufs):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            enqueue(b, torch.cuda.current_stream().cuda_stream)
        graphs.append(g)
    # eager work on a stream that owns nothing: must still find a region (and give the right bits)
    eager = [buffers(40 + i) for i in range(4)]
    for rep in range(3):
        for b in bufs:
            for t in b[3] + b[4]:
                t.zero_()
            for c in b[5]:
                c.fill_(-1)
        torch.cuda.synchronize()
        for g in graphs:
            g.replay()
        for b in eager:
            enqueue(b, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        for i, (b, e) in enumerate(zip(bufs, eager)):
            for key in (3, 4, 5):
                for x, y in zip(b[key], e[key]):
                    assert torch.equal(x.view(torch.uint8), y.view(torch.uint8)), f"replay {rep}, graph {i}, buffer {key}"
        assert int(eager[0][5][0][:, 0].abs().sum().item()) != 0
    del graphs
    torch.cuda.synchronize()
    for s in streams:
        ew.ew_scratch_release(s.cuda_stream)
    for s, b in zip(streams, bufs):           # and after the release everything still works
        with torch.cuda.stream(s):
            enqueue(b, s.cuda_stream)
    torch.cuda.synchronize()
    for b, e in zip(bufs, eager):
        for x, y in zip(b[5], e[5]):
            assert torch.equal(x, y)
    plan.close()
