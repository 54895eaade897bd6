#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

One step = one pass over one DP group's state (all four arrays P/W/M/V resident in HBM):
  a1 plan      ew_plan_bounds + ew_plan_upload (host, counted in the step time)
  a2 snapshot  ew_snapshot of every old rank's partition (copy + per-MiB checksums)
  a3 verify    ew_verify of the snapshots that replace failed ranks
  a4 pack      ew_pack   (non-local segments -> staging arena)
  a6+a7        ew_unpack_snapshot: arena + local segments -> new shards, their snapshot copies and
               the checksums of the new shards, every element read once
               (--unfused: ew_unpack, then ew_snapshot of every new rank's partition)
The 70B stage does not fit 288 GB with all four arrays resident (299 GB): there the step is measured
one state array at a time (that array resident before its own timed steps) and the four are summed.
`value` is the algorithmic bytes (read + written) of the kernels as run divided by the step's wall
time; `ms_per_step` is the figure that shows what fusing a6 and a7 saves.  The path not chosen for
the headline is timed too, after the timed region, and reported under "other_path".

After the timed region the default run (7b_stage) also measures, each on its own and briefly, the
other named workloads -- tiny (latencies), one 7B rank shard's snapshot + verify, the 13B stage and
the 70B stage -- and reports them under "workloads" (--no-workloads skips this).  The CPU baseline
is the oracle alone: nothing of the library is called inside it.

Prints ONE JSON line.  --gpus above 1 is refused: this build is one GPU only.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E peak

KERNEL_OF = {"snapshot_old": "ew_cksum_slots_kernel<copy> (+ ew_fold_kernel) = ew_snapshot",
             "snapshot_new": "ew_cksum_slots_kernel<copy> (+ ew_fold_kernel) = ew_snapshot",
             "verify": "ew_cksum_kernel<read-only> (+ ew_compare_kernel) = ew_verify",
             "pack": "ew_segcopy_kernel = ew_pack", "unpack": "ew_segcopy_kernel = ew_unpack",
             "unpack_snapshot": "ew_unpack_snap_kernel (+ ew_fold_tiles_kernel) = ew_unpack_snapshot"}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="7b_stage",
                    choices=["tiny", "7b_stage", "7b_rank_snapshot", "13b_stage", "70b_stage"],
                    help="70b_stage does not fit 288 GB with all four arrays resident: it is measured one "
                         "array at a time (each array resident before its own timed steps) and summed")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-units", type=int, default=8192)
    ap.add_argument("--unfused", action="store_true",
                    help="headline path runs a6 (ew_unpack) and a7 (ew_snapshot) separately")
    ap.add_argument("--no-other-path", action="store_true", help="do not time the path that is not the headline")
    ap.add_argument("--no-migration", action="store_true", help="skip the layer-migration comparison (Sec. 6.3)")
    ap.add_argument("--no-placement-trial", action="store_true",
                    help="keep the plain allocation of the new shards and their snapshot copies instead of the best of a few")
    ap.add_argument("--no-workloads", action="store_true",
                    help="skip the brief measurements of the other named workloads after the timed region")
    ap.add_argument("--no-grad-snapshot", action="store_true",
                    help="skip the gradient-shipping snapshot measurement (Sec. 5.1)")
    return ap.parse_args()


def log(msg):
    """Progress on stderr (stdout carries the one JSON line): long runs must not look hung."""
    print(f"bench: {msg}", file=sys.stderr, flush=True)


def read_traffic(kernel_key):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary
    (FETCH_SIZE / WRITE_SIZE runs); None when no summary for this kernel and workload exists."""
    path = os.path.join(ROOT, "profiles", "pmc_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        t = line.split()
        if len(t) >= 2 and t[0] == kernel_key:
            try:
                return float(t[1])
            except ValueError:
                return None
    return None


def merge_paths(parts):
    """Sums the per-array measurements of one path."""
    out = {"ms_per_step": 0.0, "plan_ms": 0.0, "step_device_ms_min": 0.0, "step_device_ms_max": 0.0,
           "phase_ms": {}, "phase_median_ms": {}, "bytes_phase": {}, "launches": {}}
    for p in parts:
        for key in ("ms_per_step", "plan_ms", "step_device_ms_min", "step_device_ms_max"):
            out[key] += p[key]
        for key in ("phase_ms", "phase_median_ms", "bytes_phase", "launches"):
            for ph, v in p[key].items():
                out[key][ph] = out[key].get(ph, 0) + v
    return out


def summarise(path, workload_name):
    """value, per-phase table and the roofline of the dominant kernel of one (merged) path."""
    phase_ms, bytes_phase, launches = path["phase_ms"], path["bytes_phase"], path["launches"]
    kernels = {}
    for ph in phase_ms:
        if phase_ms[ph] > 0:
            gbs = bytes_phase[ph] / phase_ms[ph] / 1e6
            kernels[ph] = {"ms": round(phase_ms[ph], 4), "ms_median": round(path["phase_median_ms"][ph], 4),
                           "launches": launches[ph], "GB": round(bytes_phase[ph] / 1e9, 4),
                           "GB/s": round(gbs, 1), "frac_of_peak": round(gbs / HBM_PEAK_GBS, 4)}
    # dominant kernel: the one whose launches take the most time in a step
    groups = {}
    for ph in phase_ms:
        g = groups.setdefault(KERNEL_OF[ph], [0.0, 0.0, 0])
        g[0] += phase_ms[ph]
        g[1] += bytes_phase[ph]
        g[2] += launches[ph]
    dom = max(groups, key=lambda k: groups[k][0])
    d_ms, d_bytes, d_launches = groups[dom]
    achieved = d_bytes / d_ms / 1e6
    roofline = {"kernel": dom, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": read_traffic(f"{dom.split()[-1]}/{workload_name}"),
                "bytes_per_launch": round(d_bytes / d_launches), "avg_launch_us": round(d_ms / d_launches * 1e3, 2)}
    step_bytes = sum(bytes_phase.values())
    return {"ms_per_step": path["ms_per_step"], "value": step_bytes / path["ms_per_step"] / 1e6,
            "step_device_ms_min": path["step_device_ms_min"], "step_device_ms_max": path["step_device_ms_max"],
            "step_GB": step_bytes / 1e9, "plan_ms": path["plan_ms"], "kernels": kernels, "roofline": roofline}


def measure(args, ew, synth, torch, w, starts, A, keep_state, steps=None, warmup=None, do_other=None, extras=True):
    """Everything that needs the state arrays `A` of workload `w` resident in HBM: the timed steps of
    the headline path, the other path, the plain-copy yardstick and the stand-alone reshard time."""
    dev = "cuda:0"
    st = torch.cuda.current_stream().cuda_stream
    bpe = sum(synth.ELEM_SIZE[a] for a in A)
    es = synth.ELEM_SIZE
    numel = w.numel
    steps = args.steps if steps is None else steps
    warmup = args.warmup if warmup is None else warmup
    do_other = (not args.no_other_path) if do_other is None else do_other
    # ---------------- setup (untimed): state resident in HBM
    plan0 = ew.ew_plan_bounds(w.old_dp, w.new_dp, w.alive_mask, starts)
    alive = [(w.alive_mask >> j) & 1 for j in range(w.old_dp)]
    old_len = [plan0.old_shard_len(j) for j in range(w.old_dp)]
    new_len = [plan0.new_shard_len(k) for k in range(w.new_dp)]
    stage_len = plan0.stage_len
    plan0.close()
    es = synth.ELEM_SIZE
    old = {a: [synth.fill(w.seed, j, a, 0, old_len[j], dev) for j in range(w.old_dp)] for a in A}
    snap = {a: [torch.empty_like(t) for t in old[a]] for a in A}
    sums = {a: [torch.zeros((ew.num_blocks(n * es[a]), 2), dtype=torch.int64, device=dev) for n in old_len] for a in A}
    stage = {a: torch.empty(stage_len, dtype=synth.TORCH_DTYPE[a], device=dev) for a in A}
    new = {a: [torch.empty(n, dtype=synth.TORCH_DTYPE[a], device=dev) for n in new_len] for a in A}
    nsnap = {a: [torch.empty_like(t) for t in new[a]] for a in A}
    nsums = {a: [torch.zeros((ew.num_blocks(n * es[a]), 2), dtype=torch.int64, device=dev) for n in new_len] for a in A}
    got = {a: [torch.zeros_like(t) for t in sums[a]] for a in A}
    n_bad = torch.zeros(1, dtype=torch.int64, device=dev)
    bad = torch.zeros(16, dtype=torch.int64, device=dev)
    diffs = torch.zeros((16, 2), dtype=torch.int64, device=dev)
    # after the failure the failed ranks' device memory is not available to pack/unpack
    old_after = {a: [t if alive[j] else None for j, t in enumerate(old[a])] for a in A}
    snap_used = {a: [None if alive[j] else t for j, t in enumerate(snap[a])] for a in A}
    torch.cuda.synchronize()
    log(f"{w.name} arrays {','.join(A)}: state resident in HBM")

    # ---------------- placement trial (set-up, untimed).  The fused kernel streams from three places at once
    # (sources, new shards, their snapshot copies), and its rate depends on which of the HBM's three 96-GiB
    # regions each of them lies in (6.2 TB/s with all three in one region, 6.3-6.4 with both written buffers in
    # one, 6.55-6.65 otherwise).  A program sees no physical addresses, so these long-lived buffers are placed
    # the way a long-running job can place them: a few candidate allocations, one fused call on each, keep the
    # best -- first for the snapshot copies, then for the new shards.
    placement = None
    set_bytes = sum(n * es[a] for a in A for n in new_len)
    if extras and not args.no_placement_trial and set_bytes >= (1 << 30):
        free_b, _ = torch.cuda.mem_get_info()
        n_extra = max(0, min(6, int((free_b - (16 << 30)) // set_bytes)))
        sets = [new, nsnap]
        for _ in range(n_extra):
            try:
                sets.append({a: [torch.empty_like(t) for t in new[a]] for a in A})
            except torch.OutOfMemoryError:   # free memory in pieces too small: make do with the sets there are
                torch.cuda.empty_cache()
                break
        tp = ew.ew_plan_bounds(w.old_dp, w.new_dp, w.alive_mask, starts)
        ew.ew_plan_upload(tp, 0, st)
        for a in A:                      # real bytes in the sources the trial reads
            for j in range(w.old_dp):
                if not alive[j]:
                    ew.ew_snapshot(old[a][j], snap[a][j], old_len[j] * es[a], sums[a][j], st)
            ew.ew_pack(tp, old_after[a], snap_used[a], stage[a], es[a], st)

        def fused_rate(shards, copies):
            ts = []
            for rep in range(4):
                p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                p0.record()
                for a in A:
                    ew.ew_unpack_snapshot(tp, stage[a], old_after[a], snap_used[a], shards[a], copies[a], nsums[a], es[a], st)
                p1.record()
                torch.cuda.synchronize()
                ts.append(p0.elapsed_time(p1))
            return round(3 * set_bytes / sorted(ts[1:])[1] / 1e6, 1)

        # set 0 = the new shards as allocated, set 1 = their copies as allocated, sets 2.. = what came after
        copies_rates = {i: fused_rate(sets[0], sets[i]) for i in range(1, len(sets))}
        ci = max(copies_rates, key=copies_rates.get)
        shards_rates = {i: (copies_rates[ci] if i == 0 else fused_rate(sets[i], sets[ci]))
                        for i in range(len(sets)) if i != ci}
        si = max(shards_rates, key=shards_rates.get)
        tp.close()
        new, nsnap = sets[si], sets[ci]
        del sets
        torch.cuda.empty_cache()
        placement = {"fused_GBps_by_copies_set": copies_rates, "copies_set": ci,
                     "fused_GBps_by_shards_set": shards_rates, "shards_set": si}
        log(f"placement trial: copies {copies_rates} -> set {ci}; shards {shards_rates} -> set {si}")

    numel = w.numel
    n_remote = stage_len
    ck_old = 16 * sum(int(t.shape[0]) for a in A for t in sums[a])
    ck_new = 16 * sum(int(t.shape[0]) for a in A for t in nsums[a])

    def phase_table(unfused):
        b = {"snapshot_old": sum(2 * n * bpe for n in old_len) + ck_old,
             "verify": sum(old_len[j] * bpe for j in w.failed),
             "pack": 2 * bpe * n_remote}
        n = {"snapshot_old": len(A) * w.old_dp, "verify": len(A) * len(w.failed), "pack": len(A)}
        if unfused:
            b["unpack"] = 2 * bpe * numel
            b["snapshot_new"] = sum(2 * x * bpe for x in new_len) + ck_new
            n.update({"unpack": len(A), "snapshot_new": len(A) * w.new_dp})
        else:
            b["unpack_snapshot"] = 3 * bpe * numel + ck_new    # read once, written twice
            n["unpack_snapshot"] = len(A)
        return b, n

    def step(unfused, record):
        ev = []

        def mark():
            if record:
                e = torch.cuda.Event(enable_timing=True)
                e.record()
                ev.append(e)

        t0 = time.perf_counter()
        plan = ew.ew_plan_bounds(w.old_dp, w.new_dp, w.alive_mask, starts)          # a1
        ew.ew_plan_upload(plan, 0, st)
        t_plan = time.perf_counter() - t0
        mark()
        for a in A:                                                                    # a2
            for j in range(w.old_dp):
                ew.ew_snapshot(old[a][j], snap[a][j], old_len[j] * es[a], sums[a][j], st)
        mark()
        for a in A:                                                                    # a3
            for j in w.failed:
                ew.ew_verify(snap[a][j], old_len[j] * es[a], sums[a][j], got[a][j], n_bad, bad, diffs, 16, st)
        mark()
        for a in A:                                                                    # a4
            ew.ew_pack(plan, old_after[a], snap_used[a], stage[a], es[a], st)
        mark()
        if unfused:
            for a in A:                                                                # a6
                ew.ew_unpack(plan, stage[a], old_after[a], snap_used[a], new[a], es[a], st)
            mark()
            for a in A:                                                                # a7
                for k in range(w.new_dp):
                    ew.ew_snapshot(new[a][k], nsnap[a][k], new_len[k] * es[a], nsums[a][k], st)
        else:
            for a in A:                                                                # a6 + a7
                ew.ew_unpack_snapshot(plan, stage[a], old_after[a], snap_used[a], new[a], nsnap[a], nsums[a], es[a], st)
        mark()
        return plan, t_plan, ev

    def run_path(unfused, steps, warmup):
        """W untimed steps, then exactly K timed steps between two device synchronisations."""
        bytes_phase, launches = phase_table(unfused)
        phases = list(bytes_phase)
        plans = [step(unfused, False)[0] for _ in range(warmup)]
        torch.cuda.synchronize()
        for p in plans:
            p.close()
        plans, records = [], []
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            p, t_plan, ev = step(unfused, True)
            plans.append(p)      # freed after the region: the kernels that use its tables are in flight
            records.append((t_plan, ev))
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        for p in plans:
            p.close()
        assert int(n_bad.item()) == 0, "verification of an intact snapshot reported bad blocks"
        phase_ms = {ph: sum(ev[i].elapsed_time(ev[i + 1]) for _, ev in records) / steps for i, ph in enumerate(phases)}
        phase_median = {ph: sorted(ev[i].elapsed_time(ev[i + 1]) for _, ev in records)[steps // 2]
                        for i, ph in enumerate(phases)}
        per_step = [ev[0].elapsed_time(ev[-1]) for _, ev in records]   # device time of each step, plan excluded
        return {"ms_per_step": elapsed / steps * 1e3, "plan_ms": sum(r[0] for r in records) / steps * 1e3,
                "step_device_ms_min": min(per_step), "step_device_ms_max": max(per_step),
                "phase_ms": phase_ms, "phase_median_ms": phase_median, "bytes_phase": bytes_phase, "launches": launches}

    # ---------------- the timed region (inside run_path): exactly K steps of the headline path
    head = run_path(args.unfused, steps, warmup)
    log(f"{w.name} arrays {','.join(A)}: {steps} timed steps done, {head['ms_per_step']:.3f} ms per step")
    other = run_path(not args.unfused, steps, 1) if do_other else None

    # yardstick (outside the timed region): the library's plain copy kernel on one fp32 rank shard,
    # i.e. what a copy with nothing else to do reaches on this GPU; these launches are also the
    # known-size dispatches (ybytes read, ybytes written) that the profiler's byte counters are
    # calibrated with
    ysrc, ydst = old[A[-1]][0], snap[A[-1]][0]
    ybytes = (old_len[0] * es[A[-1]]) & ~15
    for _ in range(3):
        ew.ew_memcpy(ysrc, ydst, ybytes, st)
    y0, y1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    y0.record()
    for _ in range(10):
        ew.ew_memcpy(ysrc, ydst, ybytes, st)
    y1.record()
    torch.cuda.synchronize()
    copy_gbs = 2 * ybytes * 10 / y0.elapsed_time(y1) / 1e6

    # time to reshard one stage on its own (outside the timed region): plan + table upload + pack +
    # unpack of all four arrays, host clock around a synchronised run, median of 7
    reshard_runs = []
    for _ in range(7 if extras else 3):
        torch.cuda.synchronize()
        r0 = time.perf_counter()
        rp = ew.ew_plan_bounds(w.old_dp, w.new_dp, w.alive_mask, starts)
        ew.ew_plan_upload(rp, 0, st)
        for a in A:
            ew.ew_pack(rp, old_after[a], snap_used[a], stage[a], es[a], st)
        for a in A:
            ew.ew_unpack(rp, stage[a], old_after[a], snap_used[a], new[a], es[a], st)
        torch.cuda.synchronize()
        reshard_runs.append((time.perf_counter() - r0) * 1e3)
        rp.close()
    reshard_only_ms = sorted(reshard_runs)[len(reshard_runs) // 2]

    # the same without the arena (holders and destinations in one address space, as on this one GPU):
    # plan + upload + ew_reshard of the four arrays, and the variant that also takes the new snapshot
    direct_runs, direct_snap_runs = [], []
    for _ in range(7 if extras else 3):
        for runs, with_snapshot in ((direct_runs, False), (direct_snap_runs, True)):
            torch.cuda.synchronize()
            r0 = time.perf_counter()
            rp = ew.ew_plan_bounds(w.old_dp, w.new_dp, w.alive_mask, starts)
            ew.ew_plan_upload(rp, 0, st)
            for a in A:
                if with_snapshot:
                    ew.ew_reshard_snapshot(rp, old_after[a], snap_used[a], new[a], nsnap[a], nsums[a], es[a], st)
                else:
                    ew.ew_reshard(rp, old_after[a], snap_used[a], new[a], es[a], st)
            torch.cuda.synchronize()
            runs.append((time.perf_counter() - r0) * 1e3)
            rp.close()
    direct_ms = sorted(direct_runs)[len(direct_runs) // 2]
    direct_snap_ms = sorted(direct_snap_runs)[len(direct_snap_runs) // 2]

    tiny_latency = None
    if w.name == "tiny":
        # cache-resident and launch bound: read these as latencies, not as fractions of HBM peak.  The
        # device part of a step (a2..a7, ~45 launches) replayed from a HIP graph vs issued call by call.
        side = torch.cuda.Stream()
        gplan = ew.ew_plan_bounds(w.old_dp, w.new_dp, w.alive_mask, starts)
        ew.ew_plan_upload(gplan, 0, side.cuda_stream)

        def device_part(s):
            for a in A:
                for j in range(w.old_dp):
                    ew.ew_snapshot(old[a][j], snap[a][j], old_len[j] * es[a], sums[a][j], s)
            for a in A:
                for j in w.failed:
                    ew.ew_verify(snap[a][j], old_len[j] * es[a], sums[a][j], got[a][j], n_bad, bad, diffs, 16, s)
            for a in A:
                ew.ew_pack(gplan, old_after[a], snap_used[a], stage[a], es[a], s)
                ew.ew_unpack_snapshot(gplan, stage[a], old_after[a], snap_used[a], new[a], nsnap[a], nsums[a], es[a], s)

        with torch.cuda.stream(side):
            device_part(side.cuda_stream)
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            device_part(torch.cuda.current_stream().cuda_stream)
        lat = {}
        for name, fn in (("eager", lambda: device_part(st)), ("graph_replay", graph.replay)):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(50):
                fn()
            torch.cuda.synchronize()
            lat[name + "_us"] = round((time.perf_counter() - t0) / 50 * 1e6, 1)
        tiny_latency = lat
        gplan.close()
    return {"head": head, "other": other, "copy_gbs": copy_gbs, "reshard_only_ms": reshard_only_ms, "direct_ms": direct_ms,
            "direct_snap_ms": direct_snap_ms, "n_remote": n_remote,
            "old_len": old_len, "keep": (old, alive) if keep_state else None, "tiny_latency": tiny_latency,
            "placement": placement}


def run_stage(args, ew, configs, synth, torch, name, steps=None, warmup=None, do_other=None, extras=True):
    """Measures one of the stage workloads (tiny, 7b, 13b, 70b) and returns the summarised paths plus
    what the callers report next to them."""
    w = configs.ALL[name]()
    starts = w.unit_starts()
    A = list(synth.ARRAYS)
    # all four arrays resident at once, except where that exceeds the GPU's memory
    residency = [[a] for a in A] if w.name == "70b_stage" else [A]
    parts = []
    for group in residency:
        parts.append(measure(args, ew, synth, torch, w, starts, group, keep_state=(len(residency) == 1),
                             steps=steps, warmup=warmup, do_other=do_other, extras=extras))
        torch.cuda.empty_cache()
    res = {"w": w, "starts": starts,
           "head": summarise(merge_paths([p["head"] for p in parts]), w.name),
           "other": None if parts[0]["other"] is None else summarise(merge_paths([p["other"] for p in parts]), w.name),
           "copy_gbs": parts[-1]["copy_gbs"],
           "reshard_only_ms": sum(p["reshard_only_ms"] for p in parts),
           "direct_ms": sum(p["direct_ms"] for p in parts),
           "direct_snap_ms": sum(p["direct_snap_ms"] for p in parts),
           "n_remote": parts[0]["n_remote"], "old_len": parts[0]["old_len"],
           "keep": parts[0]["keep"], "tiny_latency": parts[0]["tiny_latency"], "placement": parts[0]["placement"]}
    return res


def rank_snapshot_measure(ew, configs, synth, torch, steps, warmup):
    """The snapshot-only workload on its own: one 7B-stage rank shard (four arrays, 3.06 GB) copied with
    per-MiB checksums (ew_snapshot), then verified (ew_verify).  One step = both, all four arrays."""
    w = configs.snapshot_7b()
    dev = "cuda:0"
    st = torch.cuda.current_stream().cuda_stream
    A, es = list(synth.ARRAYS), synth.ELEM_SIZE
    src = {a: synth.fill(w.seed, 0, a, 0, w.numel, dev) for a in A}
    dst = {a: torch.empty_like(src[a]) for a in A}
    ck = {a: torch.zeros((ew.num_blocks(w.numel * es[a]), 2), dtype=torch.int64, device=dev) for a in A}
    got = {a: torch.zeros_like(ck[a]) for a in A}
    n_bad = torch.zeros(1, dtype=torch.int64, device=dev)
    bad = torch.zeros(16, dtype=torch.int64, device=dev)
    diffs = torch.zeros((16, 2), dtype=torch.int64, device=dev)
    nbytes = sum(w.numel * es[a] for a in A)
    rec = []

    def step(record):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)] if record else None
        if record:
            ev[0].record()
        for a in A:
            ew.ew_snapshot(src[a], dst[a], w.numel * es[a], ck[a], st)
        if record:
            ev[1].record()
        for a in A:
            ew.ew_verify(dst[a], w.numel * es[a], ck[a], got[a], n_bad, bad, diffs, 16, st)
        if record:
            ev[2].record()
            rec.append(ev)

    for _ in range(warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step(True)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    assert int(n_bad.item()) == 0
    snap_ms = sum(e[0].elapsed_time(e[1]) for e in rec) / steps
    ver_ms = sum(e[1].elapsed_time(e[2]) for e in rec) / steps
    ck_bytes = 16 * sum(int(ck[a].shape[0]) for a in A)
    return {"w": w, "ms_per_step": ms, "step_bytes": 3 * nbytes + ck_bytes,
            "kernels": {"snapshot": {"ms": round(snap_ms, 4), "launches": 4, "GB": round((2 * nbytes + ck_bytes) / 1e9, 4),
                                     "GB/s": round((2 * nbytes + ck_bytes) / snap_ms / 1e6, 1),
                                     "frac_of_peak": round((2 * nbytes + ck_bytes) / snap_ms / 1e6 / HBM_PEAK_GBS, 4)},
                        "verify": {"ms": round(ver_ms, 4), "launches": 4, "GB": round(nbytes / 1e9, 4),
                                   "GB/s": round(nbytes / ver_ms / 1e6, 1),
                                   "frac_of_peak": round(nbytes / ver_ms / 1e6 / HBM_PEAK_GBS, 4)}}}


def compact(res):
    """What the "workloads" block keeps of one stage workload."""
    h, w = res["head"], res["w"]
    out = {"note": w.note, "state_GB": round(14 * w.numel / 1e9, 3), "remote_fraction": round(res["n_remote"] / w.numel, 4),
           "ms_per_step": round(h["ms_per_step"], 3), "GBps": round(h["value"], 1),
           "frac_of_hbm_peak": round(h["value"] / HBM_PEAK_GBS, 4), "plan_ms": round(h["plan_ms"], 3),
           "reshard_one_stage_ms": round(res["reshard_only_ms"], 3),
           "reshard_without_arena_ms": round(res["direct_ms"], 3),
           "kernel_GBps": {ph: k["GB/s"] for ph, k in h["kernels"].items() if k["GB"] > 0},
           "dominant_kernel": {"kernel": h["roofline"]["kernel"].split()[0], "GBps": h["roofline"]["achieved"],
                               "frac": h["roofline"]["frac"], "avg_launch_us": h["roofline"]["avg_launch_us"]}}
    if w.name == "70b_stage":
        out["residency"] = "one state array at a time (299 GB do not fit 288 GB); the four are summed"
    return out


def oracle_remote_elems(o_lay, starts, old_dp, new_dp, alive_mask):
    """Elements that change rank (the arena's length), from the oracle's layout functions alone."""
    import numpy as np
    alive = o_lay.alive_list(old_dp, alive_mask)
    nro = o_lay.new_rank_of(old_dp, new_dp, alive)
    lens, counts = np.unique(np.diff(np.asarray(starts, dtype=np.int64)), return_counts=True)
    total = 0
    for L, c in zip(lens.tolist(), counts.tolist()):
        nb = o_lay.piece_bounds(L, new_dp)
        per_unit = 0
        for h in range(old_dp):
            for lo, hi, _owner in o_lay.held_ranges(L, h, old_dp, alive):
                for k in range(new_dp):
                    if nro[h] != k:
                        per_unit += max(0, min(hi, nb[k + 1]) - max(lo, nb[k]))
        total += per_unit * c
    return total


def cpu_baseline(w, starts, host, n_units, threads):
    """One pass of the hot path by the CPU oracle over the first n_units units: snapshot + checksum of
    every old partition, verify of the failed ranks' snapshots, reconstruct + slice, snapshot +
    checksum of the result.  Nothing of the library is called.  threads > 1 runs the state arrays side
    by side (numpy releases the interpreter lock in its copies and reductions)."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    from oracle import checksum as o_ck
    from oracle import layout as o_lay
    s_starts = np.asarray(starts[:n_units + 1], dtype=np.int64)
    al = o_lay.alive_list(w.old_dp, w.alive_mask)

    def one_array(a):
        n = 0
        snaps_h = [h.copy() for h in host[a]]                         # a2: copy ...
        cks = [o_ck.block_checksums(h) for h in snaps_h]              # ... + checksum
        n += sum(2 * h.nbytes for h in host[a])
        for j in w.failed:                                            # a3
            bad_b, _ = o_ck.verify(snaps_h[j], cks[j])
            assert len(bad_b) == 0
            n += snaps_h[j].nbytes
        new_h = o_lay.reshard([h if al[j] else None for j, h in enumerate(host[a])],   # a4 + a6
                              [None if al[j] else s for j, s in enumerate(snaps_h)],
                              w.old_dp, w.new_dp, w.alive_mask, s_starts)
        nsn = [h.copy() for h in new_h]                               # a7
        _ = [o_ck.block_checksums(h) for h in nsn]
        n += sum(2 * h.nbytes for h in new_h)
        return n

    c0 = time.perf_counter()
    if threads > 1:
        with ThreadPoolExecutor(max_workers=threads) as pool:
            cpu_bytes = sum(pool.map(one_array, list(host)))
    else:
        cpu_bytes = sum(one_array(a) for a in host)
    cpu_s = time.perf_counter() - c0
    # pack + unpack traffic of the sample under the byte accounting of the unfused GPU path
    bpe = sum(h[0].itemsize for h in host.values())
    cpu_bytes += 2 * bpe * (int(s_starts[-1]) + oracle_remote_elems(o_lay, s_starts, w.old_dp, w.new_dp, w.alive_mask))
    return cpu_bytes, cpu_s


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (all simulated DP ranks live in one MI355X's HBM); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2510_00606_amd as ew
    from paper_2510_00606_amd import configs, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU fallback", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    st = torch.cuda.current_stream().cuda_stream
    A = list(synth.ARRAYS)

    if args.workload == "7b_rank_snapshot":
        r = rank_snapshot_measure(ew, configs, synth, torch, args.steps, args.warmup)
        w = r["w"]
        dom = max(r["kernels"], key=lambda k: r["kernels"][k]["ms"])
        k = r["kernels"][dom]
        print(json.dumps({
            "metric": "reshard+snapshot GB/s on one MI355X and % of HBM peak; time to reshard one stage",
            "value": round(r["step_bytes"] / r["ms_per_step"] / 1e6, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": round(r["ms_per_step"], 3), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "u64", "data": "synthetic",
            "config": {"workload": w.name, "note": w.note, "numel": w.numel, "state_bytes": 14 * w.numel,
                       "arrays": "bf16 P + fp32 W, M, V"},
            "path": "ew_snapshot of the four arrays, then ew_verify of the four copies",
            "kernels": r["kernels"],
            "roofline": {"kernel": {"snapshot": KERNEL_OF["snapshot_old"], "verify": KERNEL_OF["verify"]}[dom], "bound": "hbm",
                         "achieved": k["GB/s"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": k["frac_of_peak"],
                         "traffic": read_traffic(f"ew_{dom}/{w.name}"),
                         "bytes_per_launch": round(k["GB"] * 1e9 / k["launches"]),
                         "avg_launch_us": round(k["ms"] / k["launches"] * 1e3, 2)},
            "cpu_baseline": None}))
        return

    res = run_stage(args, ew, configs, synth, torch, args.workload)
    w, starts, head, other = res["w"], res["starts"], res["head"], res["other"]
    numel = w.numel
    n_remote, old_len = res["n_remote"], res["old_len"]
    old, alive = res["keep"] if res["keep"] else (None, None)

    names = {True: "unfused (ew_unpack, then ew_snapshot of the new shards)",
             False: "fused (ew_unpack_snapshot also writes the new shards' snapshots and checksums)"}
    out = {
        "metric": "reshard+snapshot GB/s on one MI355X and % of HBM peak; time to reshard one stage",
        "value": round(head["value"], 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(head["ms_per_step"], 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u64", "data": "synthetic",
        "config": {"workload": w.name, "note": w.note, "numel": numel, "state_bytes": 14 * numel, "old_dp": w.old_dp,
                   "new_dp": w.new_dp, "failed": w.failed, "units": int(len(starts) - 1),
                   "remote_fraction": round(n_remote / numel, 4), "arrays": "bf16 P + fp32 W, M, V"},
        "frac_of_hbm_peak": round(head["value"] / HBM_PEAK_GBS, 4),
        "step_device_ms_min_max": [round(head["step_device_ms_min"], 3), round(head["step_device_ms_max"], 3)],
        "path": names[args.unfused],
        "reshard_one_stage_ms": round(res["reshard_only_ms"], 3),
        "reshard_useful_GBps": round(14 * numel / res["reshard_only_ms"] / 1e6, 1),
        "reshard_without_arena": {
            "note": "ew_reshard: every segment pulled straight from its holder's buffer, for ranks in one address "
                    "space (outside `value`, which keeps the pack -> arena -> unpack path)",
            "reshard_ms": round(res["direct_ms"], 3), "GBps": round(28 * numel / res["direct_ms"] / 1e6, 1),
            "reshard_plus_new_snapshot_ms": round(res["direct_snap_ms"], 3),
            "reshard_plus_new_snapshot_GBps": round(42 * numel / res["direct_snap_ms"] / 1e6, 1)},
        "plan_ms": round(head["plan_ms"], 3),
        "step_GB": round(head["step_GB"], 3),
        "kernels": head["kernels"],
        "plain_copy_GBps": round(res["copy_gbs"], 1),
        "roofline": head["roofline"],
    }
    if res["placement"] is not None:
        out["placement_trial"] = dict(res["placement"], note=(
            "set-up, before the timed region: up to six more sets of new-shard-sized buffers are allocated behind the "
            "plain allocation (set 0 = new shards, set 1 = their snapshot copies); one ew_unpack_snapshot of the four "
            "arrays is timed with each set as the copies, the fastest is kept, then the same for the new shards; the rest "
            "is freed.  The kernel's rate depends on which 96-GiB regions of the HBM its three streams lie in, which a "
            "program cannot see"))
    if res["tiny_latency"] is not None:
        out["tiny_step_latency"] = res["tiny_latency"]
    if other is not None:
        out["other_path"] = {"path": names[not args.unfused], "ms_per_step": round(other["ms_per_step"], 3),
                             "value": round(other["value"], 1), "step_GB": round(other["step_GB"], 3),
                             "kernels": other["kernels"]}

    # ---------------- CPU baseline: the oracle as it stands on a bounded sample; nothing of the library is called
    if not args.no_cpu_baseline and old is None:
        out["cpu_baseline"] = None   # measured at the workloads whose state is resident all at once (default: 7b_stage)
    if not args.no_cpu_baseline and old is not None:
        from oracle import layout as o_lay
        n_units = min(args.cpu_sample_units, len(starts) - 1)
        s_starts = starts[:n_units + 1].astype(np.int64)
        s_numel = int(s_starts[-1])
        s_old_len = o_lay.shard_lengths(s_starts, w.old_dp)
        host = {a: [synth.to_numpy_bits(old[a][j][:s_old_len[j]]) for j in range(w.old_dp)] for a in A}
        torch.cuda.synchronize()
        log("CPU oracle baseline on one core ...")
        cpu_bytes, cpu_s = cpu_baseline(w, starts, host, n_units, 1)
        log(f"CPU oracle baseline: {cpu_s:.1f} s")
        out["cpu_baseline"] = {
            "value": round(cpu_bytes / cpu_s / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"first {n_units} of {len(starts) - 1} units of {w.name} ({s_numel} elements, all four arrays): "
                      f"numpy oracle snapshot+checksum, verify, reconstruct+slice, snapshot+checksum of the result, "
                      f"bytes counted as for the unfused GPU path; {cpu_s:.1f} s on one host core",
        }
        cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
        threads = min(len(A), cores)
        if threads > 1:   # the same oracle, the four state arrays side by side
            mt_bytes, mt_s = cpu_baseline(w, starts, host, n_units, threads)
            out["cpu_baseline"]["all_cores_variant"] = {
                "value": round(mt_bytes / mt_s / 1e9, 3), "unit": "GB/s", "cores": threads, "cores_available": cores,
                "seconds": round(mt_s, 2), "note": "one host thread per state array (the oracle reshards an array as a whole)"}
        del host
        # the tiny workload by the same oracle (cache-sized: a latency, like the GPU's)
        tw = configs.tiny()
        t_starts = tw.unit_starts()
        t_len = o_lay.shard_lengths(t_starts.astype(np.int64), tw.old_dp)
        t_host = {a: [synth.to_numpy_bits(synth.fill(tw.seed, j, a, 0, t_len[j], "cpu")) for j in range(tw.old_dp)] for a in A}
        t_bytes, t_s = min((cpu_baseline(tw, t_starts, t_host, len(t_starts) - 1, 1) for _ in range(5)), key=lambda r: r[1])
        out["cpu_baseline"]["tiny"] = {"ms_per_step": round(t_s * 1e3, 3), "value": round(t_bytes / t_s / 1e9, 3),
                                       "unit": "GB/s", "cores": 1}

    del old, res
    torch.cuda.empty_cache()
    # ---------------- the other named workloads, briefly, each on its own (outside the timed region)
    if not args.no_workloads and w.name == "7b_stage":
        wl = {}
        t = run_stage(args, ew, configs, synth, torch, "tiny", steps=20, warmup=3, do_other=False, extras=False)
        wl["tiny"] = {"note": t["w"].note + "; cache resident and launch bound: latencies, not HBM fractions",
                      "ms_per_step": round(t["head"]["ms_per_step"], 4), "plan_ms": round(t["head"]["plan_ms"], 4),
                      "reshard_one_stage_ms": round(t["reshard_only_ms"], 4), "device_part_latency": t["tiny_latency"]}
        del t
        log("workloads: tiny done")
        r = rank_snapshot_measure(ew, configs, synth, torch, 10, 2)
        wl["7b_rank_snapshot"] = {"note": r["w"].note, "state_GB": round(14 * r["w"].numel / 1e9, 3),
                                  "ms_per_step": round(r["ms_per_step"], 4),
                                  "GBps": round(r["step_bytes"] / r["ms_per_step"] / 1e6, 1), "kernels": r["kernels"]}
        del r
        torch.cuda.empty_cache()
        for name, k in (("13b_stage", 5), ("70b_stage", 3)):
            t = run_stage(args, ew, configs, synth, torch, name, steps=k, warmup=1, do_other=False, extras=False)
            wl[name] = compact(t)
            log(f"workloads: {name} done")
            del t
            torch.cuda.empty_cache()
        out["workloads"] = wl

    # ---------------- layer migration, contiguous vs interleaved assignment (Sec. 6.3); not part of `value`
    if not args.no_migration and w.name != "tiny":
        torch.cuda.empty_cache()
        out["layer_migration"] = migration_compare(ew, configs, synth, torch, st, dev)
    if not args.no_grad_snapshot and w.name != "tiny":
        torch.cuda.empty_cache()
        out["gradient_snapshot"] = grad_snapshot_measure(ew, synth, torch, st, dev, old_len[0], w.seed)
    print(json.dumps(out))


def grad_snapshot_measure(ew, synth, torch, st, dev, n, seed):
    """One rank's partition (n elements): the owner's Adam step on the live shard, the gradient shard
    shipped device -> device -> pinned host, and the replay of the step on a host-resident snapshot
    (Sec. 5.1, Fig. 6).  Not part of `value`."""
    import numpy as np
    live = {a: synth.fill(seed, 0, a, 0, n, dev) for a in ("W", "M", "V")}
    live["V"] = live["V"].abs()
    live["P"] = live["W"].to(torch.bfloat16)
    snap = {a: live[a].cpu().clone() for a in live}
    g = synth.fill(seed + 1, 7, "M", 0, n, dev) * 0.05
    peer = torch.empty_like(g)
    host_g = torch.empty(n, dtype=torch.float32).pin_memory()
    res = {"elements": n, "gradient": "fp32"}
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    t_step, t_d2d, t_d2h, t_host = [], [], [], []
    for t in range(1, 5):
        h = ew.ew_adam_hyper(3e-4, 0.9, 0.95, 1e-8, 0.1, t)
        ev[0].record()
        ew.ew_adam_step(live["P"], live["W"], live["M"], live["V"], g, 4, n, h, st)
        ev[1].record()
        ew.ew_grad_ship(g, peer, None, 4 * n, st)
        ev[2].record()
        ew.ew_grad_ship(peer, None, host_g, 4 * n, st)
        ev[3].record()
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        ew.ew_adam_replay_host(snap["P"], snap["W"], snap["M"], snap["V"], host_g, 4, n, h, 0)
        c1 = time.perf_counter()
        if t > 1:
            t_step.append(ev[0].elapsed_time(ev[1]))
            t_d2d.append(ev[1].elapsed_time(ev[2]))
            t_d2h.append(ev[2].elapsed_time(ev[3]))
            t_host.append((c1 - c0) * 1e3)
    same = all(torch.equal(live[a].cpu().view(torch.int16), snap[a].view(torch.int16)) for a in live)
    med = lambda x: sorted(x)[len(x) // 2]
    res.update({
        "snapshot_equals_live_after_4_steps": bool(same),
        "adam_step_ms": round(med(t_step), 3), "adam_step_GBps": round(30 * n / med(t_step) / 1e6, 1),
        "adam_step_frac_of_hbm_peak": round(30 * n / med(t_step) / 1e6 / HBM_PEAK_GBS, 4),
        "grad_d2d_ms": round(med(t_d2d), 3), "grad_d2h_ms": round(med(t_d2h), 3),
        "grad_d2h_GBps": round(4 * n / med(t_d2h) / 1e6, 1),
        "host_replay_ms": round(med(t_host), 1), "host_replay_GBps": round(30 * n / med(t_host) / 1e6, 1),
        "host_threads": os.cpu_count() if not hasattr(os, "sched_getaffinity") else len(os.sched_getaffinity(0)),
        "bytes_shipped_per_element": 4, "bytes_of_state_per_element": 14,
        "note": "shipping the fp32 gradient moves 3.5x less than the 14 B/element state kept here "
                "(4x against a 16 B/element state with an fp32 parameter copy; 7x with bf16 gradients)",
    })
    return res


def migration_compare(ew, configs, synth, torch, st, dev):
    """Moves one Llama-7B-shaped layer between two 4-layer stages at DP 8 under both ZeRO assignments,
    all four state arrays, and reports what crosses between ranks (the arena) and how long the send
    side (ew_pack) and the whole move (ew_pack + ew_unpack) take on this GPU."""
    D = 8
    wl = configs.Workload("migrate", 9, configs.stage_tensors(4096, 11008, 4), D, D, 0xFF, 262144, snap_to_tensors=True)
    starts = wl.unit_starts()
    per_layer = (len(starts) - 1) // 4
    layer_elems = int(starts[per_layer])
    res = {"stage": "2 stages x 4 Llama-7B-shaped layers, DP 8, one layer (|O_i| = %d elements x 14 B) moves" % layer_elems}
    for name, assignment in (("interleaved", ew.EW_ASSIGN_INTERLEAVED), ("contiguous", ew.EW_ASSIGN_CONTIGUOUS)):
        plan = ew.ew_plan_migrate(assignment, D, starts, starts, per_layer)
        ew.ew_plan_upload(plan, 0, st)
        pack_ms = unpack_ms = 0.0
        for a in synth.ARRAYS:
            esz = synth.ELEM_SIZE[a]
            dt = synth.TORCH_DTYPE[a]
            old = [synth.fill(wl.seed, r, a, 0, plan.old_shard_len(r), dev) for r in range(2 * D)]
            new = [torch.empty(plan.new_shard_len(r), dtype=dt, device=dev) for r in range(2 * D)]
            arena = torch.empty(max(plan.stage_len, 1), dtype=dt, device=dev)
            tp, tu = [], []
            for rep in range(4):
                e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
                e[0].record()
                ew.ew_pack(plan, old, None, arena, esz, st)
                e[1].record()
                ew.ew_unpack(plan, arena, old, None, new, esz, st)
                e[2].record()
                torch.cuda.synchronize()
                if rep:
                    tp.append(e[0].elapsed_time(e[1]))
                    tu.append(e[1].elapsed_time(e[2]))
            pack_ms += sorted(tp)[1]
            unpack_ms += sorted(tu)[1]
            del old, new, arena
            torch.cuda.empty_cache()
        pairs = sum(1 for h in range(2 * D) for k in range(2 * D) if plan.pair_len(h, k))
        cross = sum(plan.pair_len(h, k) for h in range(D) for k in range(D, 2 * D))
        res[name] = {"messages": pairs, "moved_between_ranks_elems": plan.stage_len, "cross_stage_elems": cross,
                     "moved_over_layer": round(plan.stage_len / layer_elems, 4),
                     "arena_GB": round(14 * plan.stage_len / 1e9, 3), "pack_ms": round(pack_ms, 3),
                     "pack_plus_unpack_ms": round(pack_ms + unpack_ms, 3)}
        plan.close()
    res["contiguous_over_interleaved_bytes"] = round(res["contiguous"]["moved_between_ranks_elems"] /
                                                     res["interleaved"]["moved_between_ranks_elems"], 3)
    res["contiguous_over_interleaved_pack_time"] = round(res["contiguous"]["pack_ms"] / res["interleaved"]["pack_ms"], 3)
    res["paper_closed_form"] = "interleaved |O_i| in D sends; contiguous |O_i| + (D-1)/2 |O_i| per stage"
    return res


if __name__ == "__main__":
    main()
