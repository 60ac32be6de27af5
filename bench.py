#!/usr/bin/env python3
"""Benchmark of the resilient ring all-reduce hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input:
r2_ring_allreduce_sim = partition of every transmission (channel state changes
included) + every fused step of the ring, for all simulated ranks.  Inputs are
resident in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--steps K] [--warmup W] [--config cfg2] [--no-cpu-baseline] [--all]
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

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, vendor figure (8 TB/s)

# Bytes per launch between L2 and the memory fabric for the dominant kernel, from two
# `rocprofv3 --pmc` runs of this script (FETCH_SIZE, then WRITE_SIZE; KiB per dispatch), each scaled
# by what the same counter reads for a plain device-to-device copy of one rank buffer in the same run
# (FETCH_SIZE reads half the copied bytes there, WRITE_SIZE all of them).  These are figures of earlier
# profiler runs, kept in the named files with their commands: NOT measured by the run that prints them
# (the JSON line says so in roofline.traffic_source).  The counters sit between L2 and the fabric and
# cannot tell HBM from the Infinity Cache.
MEASURED_TRAFFIC = {
    ("cfg2", "sum"): (int((131113.5 * (131072.0 / 65551.0) + 262152.2 * (131072.0 / 131072.0)) * 1024),
                      "profiles/ring_step_sum_bf16_cfg2_pmc.md"),
    ("cfg3", "sum"): (int((131114.5 * (262144.0 / 131087.6) + 262160.0 * (262144.0 / 262144.0)) * 1024),
                      "profiles/ring_step_sum_f32_cfg3_pmc.md"),
    ("cfg4", "sum"): (int((65611.5 * (65536.0 / 32781.3) + 131074.2 * (65536.0 / 65536.0)) * 1024),
                      "profiles/ring_step_sum_bf16_cfg4_pmc.md"),
}

OTHER_CONFIGS = ("cfg1", "cfg3", "cfg4", "cfg5_tok1", "cfg5_tok16", "cfg5_tok64", "cfg5_tok256")


def _workload(name: str):
    import workloads as wl

    if name.startswith("cfg5"):
        tok = int(name.split("tok")[1]) if "tok" in name else 256
        return wl.cfg5(tok)
    return {"cfg1": wl.cfg1, "cfg2": wl.cfg2, "cfg3": wl.cfg3, "cfg4": wl.cfg4}[name]()


def _desc(r2, w, window=0, schedule=0):
    dt = r2.F32 if w.dtype == "f32" else r2.BF16
    ph = {"ar": r2.PHASE_AR, "rs": r2.PHASE_RS, "ag": r2.PHASE_AG}[w.phases]
    return r2.SimDesc(w.R, w.S, w.C, w.align, w.N, dt, ph, window, schedule)


def _to_device(torch, np, x):
    return torch.from_numpy(x.view(np.int16) if x.dtype == np.uint16 else x).cuda()


class Runner:
    """Device state of one workload: pristine inputs, working buffers, workspace."""

    def __init__(self, r2, torch, np, w, xs, window=0, schedule=0):
        self.r2, self.torch, self.w = r2, torch, w
        self.desc = _desc(r2, w, window, schedule)
        self.fused = r2.r2_sim_resolve_schedule(self.desc, w.epochs) == r2.SCHED_FUSED
        self.pristine = [_to_device(torch, np, x) for x in xs]
        self.bufs = [p.clone() for p in self.pristine]
        self.ws = torch.empty(r2.r2_sim_workspace_bytes(self.desc), dtype=torch.uint8, device="cuda")
        self.J = r2.r2_sim_num_steps(self.desc)
        self.P = r2.r2_sim_num_passes(self.desc)
        self.call = r2.SimCall(self.desc, self.bufs, w.epochs, self.ws)  # arguments marshalled once

    def _fused_times(self, reps: int):
        """Fused-column schedule: a run is one launch per stretch of steps between channel-state
        changes, a few microseconds each, so a pair of events round a single launch would mostly time
        the host.  Whole runs are issued back to back between one pair of events instead (in place,
        as in time_steps); the figure is the average per launch, dispatch gaps included."""
        torch = self.torch
        segs = _fused_segments(self.w)
        n = max(20 * reps, 100)
        self.restore()
        for _ in range(3):
            self.step()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            self.step()
        e1.record()
        torch.cuda.synchronize()
        return {"fused": (e0.elapsed_time(e1) / (n * len(segs)), n * len(segs))}

    def graph_seconds_per_op(self, ops_per_graph: int = 100, replays: int = 100) -> float:
        """The same back-to-back ops captured once into a HIP graph and replayed: what a serving loop
        that captures its launch-bound inner loop pays per op (the entry points only enqueue kernels
        on the caller's stream, so they can be captured)."""
        torch, r2 = self.torch, self.r2
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            call = r2.SimCall(self.desc, self.bufs, self.w.epochs, self.ws)  # bound to the capturing stream
            for _ in range(ops_per_graph):
                call.run()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / (ops_per_graph * replays)

    def restore(self):
        for b, p in zip(self.bufs, self.pristine):
            b.copy_(p)

    def step(self):
        self.call.run()

    def time_steps(self, steps: int, warmup: int) -> float:
        """Seconds for `steps` back-to-back passes (in place: values grow by R per all-reduce, which
        changes no timing since the path has no data-dependent branch)."""
        torch = self.torch
        for _ in range(warmup):
            self.step()
        self.restore()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    def kernel_times(self, reps: int):
        """Average launch duration in ms per kind of fused step (the median over `reps` runs of each
        run's average), the runs driven launch by launch in the order r2_ring_allreduce_sim uses.
        Steps of one kind are consecutive within a pass (send | sum ... | copy ... | last); each such
        group is bracketed by one pair of HIP
        events, recorded on the stream the kernels run on, so the figure holds the kernels and the
        dispatch gaps between them, as in the real run.  Returns {kind: (avg_ms, launches)}."""
        torch, r2 = self.torch, self.r2
        if self.fused:
            return self._fused_times(reps)
        kinds = [_step_units(self.w, j)[0] for j in range(self.J)]
        groups = []  # (kind, first step, last step)
        for j, k in enumerate(kinds):
            if groups and groups[-1][0] == k:
                groups[-1][2] = j
            else:
                groups.append([k, j, j])
        per_rep = {}  # kind -> [average ms per launch in each repetition]
        count = {}
        for _ in range(reps):
            self.restore()
            r2.r2_sim_prepare(self.desc, self.w.epochs, self.ws)
            pairs = []
            for p in range(self.P):
                for k, j0, j1 in groups:
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    for j in range(j0, j1 + 1):
                        r2.r2_sim_step(self.desc, self.bufs, p, j, self.ws)
                    e1.record()
                    pairs.append((k, j1 - j0 + 1, e0, e1))
            torch.cuda.synchronize()
            total, n_launch = {}, {}
            for k, n, e0, e1 in pairs:
                total[k] = total.get(k, 0.0) + e0.elapsed_time(e1)
                n_launch[k] = n_launch.get(k, 0) + n
            for k in total:
                per_rep.setdefault(k, []).append(total[k] / n_launch[k])
                count[k] = count.get(k, 0) + n_launch[k]
        # the median repetition: one stall of the host or the box inside a repetition (seen: a single
        # event pair of tens of milliseconds) must not become the figure
        return {k: (sorted(v)[len(v) // 2], count[k]) for k, v in per_rep.items()}


def _fused_segments(w):
    """The step ranges the library launches in the fused schedule: a channel-state change at step c
    of some slab ends a launch before step c and before step c+1."""
    T = w.transmissions_per_slab
    starts = {e[0] % T for e in w.epochs[1:] if e[0] < w.S * T and e[0] % T != 0}
    cuts = sorted({j for c in starts for j in (c, c + 1) if j < T})
    edges = [0] + cuts + [w.steps_per_slab]
    return list(zip(edges[:-1], edges[1:]))


def _step_units(w, j):
    """(kernel kind, ring-chunk units of traffic per rank) of fused step j."""
    J = w.steps_per_slab
    if j == 0:
        return "send", 2
    last = j == J - 1
    summing = w.phases == "rs" or (w.phases == "ar" and j <= w.R - 1)
    if summing:
        return ("sum_last", 3) if last else ("sum", 4)
    return ("copy_last", 2) if last else ("copy", 3)


def _cpu_baseline(w, xs, gpu_outs, np):
    """The oracle's step-by-step ring on the host, on the same inputs: single thread and all threads.
    Also the correctness check of the GPU result of one pass."""
    import oracle

    odt = oracle.F32 if w.dtype == "f32" else oracle.BF16
    oph = {"ar": oracle.PHASE_AR, "rs": oracle.PHASE_RS, "ag": oracle.PHASE_AG}[w.phases]
    all_threads = oracle.threads()
    res = {}
    bufs = None
    for th in (all_threads, 1):
        oracle.set_threads(th)
        bufs = [x.copy() for x in xs]
        t0 = time.perf_counter()
        oracle.ring_sim(bufs, odt, w.S, w.C, w.align, list(w.epochs), oph, stage_fill=0)
        res[th] = time.perf_counter() - t0
        if all_threads == 1:
            break
    oracle.set_threads(all_threads)
    ok = all(np.array_equal(a, b) for a, b in zip(bufs, gpu_outs))
    return {
        "value": round(w.algorithmic_bytes / res[all_threads] / 1e9, 3),
        "unit": "GB/s",
        "cores": all_threads,
        "kind": "oracle",
        "sample": f"the whole {w.name} workload once (step-by-step oracle ring, {w.algorithmic_bytes} algorithmic bytes)",
        "seconds": round(res[all_threads], 3),
        "single_thread_GBps": round(w.algorithmic_bytes / res[1] / 1e9, 3),
        "single_thread_seconds": round(res[1], 3),
    }, ok


def _matches_definition(w, xs, gpu_outs, np):
    """Part of the cpu_baseline leg: the GPU result of one pass from pristine inputs against the
    oracle's result by plain definition (the left fold in ring order), every element of every rank."""
    import oracle

    odt = oracle.F32 if w.dtype == "f32" else oracle.BF16
    oph = {"ar": oracle.PHASE_AR, "rs": oracle.PHASE_RS, "ag": oracle.PHASE_AG}[w.phases]
    want = oracle.expected(xs, odt, w.S, oph)
    return all(np.array_equal(a, b) for a, b in zip(want, gpu_outs))


def _dominant(run, w, reps):
    """The dominant kernel of a run on the step schedule: the reducing step that also stages.
    Returns (kind, average launch ms, launches timed, algorithmic bytes per launch, all kinds)."""
    ktimes = run.kernel_times(reps)
    dom = "sum" if "sum" in ktimes else "copy"
    units = 4 if dom == "sum" else 3
    avg_ms, launches = ktimes[dom]
    # one fused step moves, for every rank and slab, one ring chunk through `units` streams; it is
    # spread over the run's passes, one launch each
    return dom, avg_ms, launches, units * w.N * w.elem_bytes / run.P, ktimes


def config_entry(r2, torch, np, wl, name, check, reps, cold_window=0):
    """One of the configurations the headline is not quoted on, in the schedule the library picks:
    whole-run time over back-to-back ops (in place), the rate of algorithmic bytes, the check of op #1
    from pristine inputs against the oracle, and on the step schedule the dominant kernel's launch."""
    w = _workload(name)
    xs = wl.make_inputs(w)
    run = Runner(r2, torch, np, w, xs)
    run.step()
    torch.cuda.synchronize()
    first = [b.cpu().numpy().view(x.dtype) for b, x in zip(run.bufs, xs)]
    ops = 10000 if name.startswith("cfg5") else (2000 if name == "cfg1" else 20)
    s = run.time_steps(ops, 3) / ops
    rate = w.algorithmic_bytes / s / 1e9
    e = {"schedule": "fused" if run.fused else "steps", "ops": ops}
    if s < 1e-3 / 4:
        e["us_per_op"] = round(s * 1e6, 2)
    else:
        e["ms_per_step"] = round(s * 1e3, 4)
    e["GBps"] = round(rate, 1)
    if run.fused:
        e["served_by"] = "cache (effective rate)"  # a fused run's stage traffic never leaves the caches
    else:
        e["pct_of_hbm_peak"] = round(100 * rate / HBM_PEAK_GBPS, 2)
        dom, avg_ms, launches, launch_bytes, _ = _dominant(run, w, reps)
        e["passes"] = run.P
        e["kernel"] = dom
        e["avg_launch_ms"] = round(avg_ms, 5)
        e["frac"] = round(launch_bytes / (avg_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)
        # the same run with pairs of half-window passes issued side by side on two streams (opt-in):
        # whole-run figures only, since launches that share the GPU have no duration of their own
        del run
        run = Runner(r2, torch, np, w, xs, schedule=r2.SCHED_STEPS_OVERLAP)
        run.step()
        torch.cuda.synchronize()
        same = all(np.array_equal(b.cpu().numpy().view(x.dtype), f) for b, x, f in zip(run.bufs, xs, first))
        so = run.time_steps(ops, 3) / ops
        e["overlap_schedule"] = {"ms_per_step": round(so * 1e3, 4), "GBps": round(w.algorithmic_bytes / so / 1e9, 1),
                                 "pct_of_hbm_peak": round(100 * w.algorithmic_bytes / so / 1e9 / HBM_PEAK_GBPS, 2),
                                 "passes": run.P, "same_result": bool(same)}
    if check:
        e["matches_oracle"] = bool(_matches_definition(w, xs, first, np))
    del run, first
    torch.cuda.empty_cache()
    cold = cold_one_pass(r2, torch, np, w, xs, cold_window, reps) if cold_window else None
    return e, cold


def cold_reduce_copy(r2, torch, dtype="bf16", chunk_mib=256, sets=4, reps=40):
    """The chunk worker with nothing cache-resident: stand-alone r2_reduce_copy (sum, both stages,
    8 channels of which 2 and 5 are down) on chunks of `chunk_mib` MiB, rotating over `sets` disjoint
    sets of buffers, so that every set's 3 x chunk bytes have been pushed out of the 256 MiB Infinity
    Cache by the others before it comes round again.  All four streams are HBM traffic.  Returns
    (average launch ms by events on the launching stream, algorithmic bytes per launch)."""
    C, align, mask = 8, 256, 0b100100
    nbytes = chunk_mib << 20
    dt = r2.BF16 if dtype == "bf16" else r2.F32
    off = r2.r2_partition([50000] * C, mask, nbytes, align)
    cap = (max(off[c + 1] - off[c] for c in range(C)) + 255) // 256 * 256
    d_off = torch.tensor(off, dtype=torch.int64, device="cuda")
    calls = []
    def filled(n):  # values of the workloads' distribution: all-zero buffers move faster through this GPU's
        t = torch.empty(n, dtype=torch.uint8, device="cuda")  # caches than any other data and would flatter the figure
        (t.view(torch.bfloat16) if dtype == "bf16" else t.view(torch.float32)).normal_(0.0, 0.02)
        return t

    for _ in range(sets):
        local = filled(nbytes)
        ins = [filled(cap) for _ in range(C)]
        outs = [filled(cap) for _ in range(C)]
        calls.append(r2.ReduceCopyCall(local, dt, r2.OP_SUM, ins, d_off, outs, d_off, C, cap, nbytes=nbytes))
    for i in range(2 * sets):
        calls[i % sets].run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(reps):
        calls[i % sets].run()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    del calls
    torch.cuda.empty_cache()
    return ms, 4 * nbytes


def plain_copy_rate(torch, mib=1024, sets=3, reps=24):
    """Context for the cold figures: what a plain device-to-device copy (torch's, one read and one write
    stream, buffers rotated so that nothing is cache-resident) reaches on this GPU.  Returns the
    fraction of the HBM peak (bytes read + bytes written over time)."""
    n = mib << 20
    src = [torch.empty(n, dtype=torch.uint8, device="cuda") for _ in range(sets)]
    dst = [torch.empty(n, dtype=torch.uint8, device="cuda") for _ in range(sets)]
    for i in range(sets):
        src[i].zero_()
        dst[i].copy_(src[i])
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(reps):
        dst[i % sets].copy_(src[i % sets])
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    del src, dst
    torch.cuda.empty_cache()
    return 2 * n / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS


def cold_one_pass(r2, torch, np, w, xs, window, reps):
    """A configuration with the stage window opened so far that it runs in one pass (cfg3: 256 MiB
    staged per step, which the next step no longer finds in the Infinity Cache).  The same sum kernel.
    Returns (average launch ms, algorithmic bytes per launch)."""
    run = Runner(r2, torch, np, w, xs, window=window, schedule=1)
    assert run.P == 1
    for _ in range(2):
        run.step()
    _, avg_ms, _, launch_bytes, _ = _dominant(run, w, reps)
    del run
    torch.cuda.empty_cache()
    return avg_ms, launch_bytes


def reduce_copy_sweep(r2, torch, out=sys.stderr):
    """Stand-alone r2_reduce_copy (sum, both stages) over chunk sizes, NCCL-tests style: C=8 channels
    with 0, 1 or 2 of them failed.  Buffers rotate over enough sets that nothing is re-used from
    cache at the large sizes; small sizes are cache- and launch-bound ("effective")."""
    C, align = 8, 256
    print("r2_reduce_copy sweep: sum + stage, 4 streams of `bytes` each; GB/s = 4*bytes/time", file=out)
    print(f"{'dtype':5s} {'failed':>6s} {'chunk bytes':>12s} {'sets':>4s} {'us/call':>10s} {'GB/s':>9s} {'% HBM peak':>10s}", file=out)
    for dtype, dt in (("bf16", r2.BF16), ("f32", r2.F32)):
        for mask in (0, 0b100, 0b100100):
            for log2 in (12, 14, 16, 18, 20, 22, 24, 26, 28, 30):
                nbytes = 1 << log2
                if dtype == "f32" and log2 in (14, 18, 22, 26):
                    continue
                off = r2.r2_partition([50000] * C, mask, nbytes, align)
                cap = max(max(off[c + 1] - off[c] for c in range(C)), 256)
                cap = (cap + 255) // 256 * 256
                sets = max(1, min(64, (1 << 30) // (4 * nbytes)))
                d_off = torch.tensor(off, dtype=torch.int64, device="cuda")
                calls = []
                def filled(n):  # not zeros: all-zero data moves faster through this GPU's caches than any other
                    t = torch.empty(max(n, 16), dtype=torch.uint8, device="cuda")
                    (t.view(torch.bfloat16) if dtype == "bf16" else t.view(torch.float32)).normal_(0.0, 0.02)
                    return t[:n]

                for _ in range(sets):
                    local = filled(nbytes)
                    ins = [filled(cap) for _ in range(C)]
                    outs = [filled(cap) for _ in range(C)]
                    calls.append(r2.ReduceCopyCall(local, dt, r2.OP_SUM, ins, d_off, outs, d_off, C, cap, nbytes=nbytes))
                reps = max(10, min(2000, (8 << 30) // (4 * nbytes)))
                for i in range(min(reps, 3 * sets)):
                    calls[i % sets].run()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for i in range(reps):
                    calls[i % sets].run()
                e1.record()
                torch.cuda.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / reps
                gbps = 4 * nbytes / us / 1e3
                print(f"{dtype:5s} {bin(mask).count('1'):6d} {nbytes:12d} {sets:4d} {us:10.2f} {gbps:9.1f} {100 * gbps / HBM_PEAK_GBPS:10.2f}",
                      file=out, flush=True)
                del calls
                torch.cuda.empty_cache()


def split_line(r2, torch, np, wl, out=sys.stderr):
    """R2CCL-AllReduce on the cfg2 shape: 8 ranks, bf16, 128 MiB per rank, rank 0 has lost half of its
    NICs (X = 0.5): the planner's share goes through partial all-reduce + broadcast."""
    w = wl.cfg2()
    R, N, C = w.R, w.N, w.C
    use, y, thr = r2.r2_split_plan(R, 1, 0.5)
    npart = r2.r2_split_partial_elems(R, 1, 1, r2.BF16, N, y)  # the share, rounded to what both rings divide into
    desc = r2.SplitDesc(R, 0, C, w.align, N, npart, r2.BF16)
    xs = wl.make_inputs(w)
    bufs = [_to_device(torch, np, x) for x in xs]
    ws = torch.empty(r2.r2_split_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    weights, mask = [50000] * C, 0b00001111
    for _ in range(3):
        r2.r2_split_allreduce_sim(desc, bufs, weights, mask, ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    n = 20
    for _ in range(n):
        r2.r2_split_allreduce_sim(desc, bufs, weights, mask, ws)
    torch.cuda.synchronize()
    s = (time.perf_counter() - t0) / n
    e = 2
    alg = ((7 * R - 6) * (N - npart) + (7 * (R - 1) - 6) * npart + 4 * R * npart) * e
    print(f"split        X=0.5 -> Y*={y:.4f} (threshold {thr:.4f}), {npart} of {N} elements partial: "
          f"{s * 1e6:10.1f} us/op  {alg / s / 1e9:9.1f} GB/s  {100 * alg / s / 1e9 / HBM_PEAK_GBPS:6.2f} % of HBM peak "
          f"({alg} algorithmic bytes)", file=out, flush=True)


def _time_calls(torch, fn, n=20, warm=3, rounds=3):
    """Seconds per call: `rounds` runs of n back-to-back calls each, the median run (one stall of the
    host or the box inside a 20-call run would otherwise be the figure)."""
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    runs = []
    for _ in range(rounds):
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        runs.append((time.perf_counter() - t0) / n)
    return sorted(runs)[len(runs) // 2]


def other_collectives_lines(r2, torch, np, wl, out=sys.stderr):
    """R2CCL-Balance on the other collectives it serves (Sec. 5, table of strategies; Sec. 8 and
    Appendix E measure some of them): reduce-scatter, all-gather, send/receive, broadcast, reduce and
    all-to-all on the cfg2 shape (8 ranks, bf16, 128 MiB per rank), one of eight channels down from
    the start.  Algorithmic bytes, in units of one rank buffer: a hop that only stages or only takes
    data moves 2, one that takes and stages onward 3 (so does a reduce hop: two reads, one write), a
    reduce-scatter step 4; all-to-all moves (R-1)/R of every buffer through the stage (4) and copies
    the own block (2)."""
    w = wl.cfg2()
    R, N, C, e = w.R, w.N, w.C, 2
    epochs = [(0, 0b00000100, [50000] * C)]
    xs = wl.make_inputs(w)
    bufs = [_to_device(torch, np, x) for x in xs]
    recv = [torch.empty_like(b) for b in bufs]
    for name, phases, S, units in (("reduce-scatter", r2.PHASE_RS, 1, (4 * R - 3) * N),
                                   ("all-gather", r2.PHASE_AG, 1, (3 * R - 2) * N),
                                   ("send/receive", r2.PHASE_SENDRECV, 8, 4 * R * N),
                                   ("broadcast", r2.PHASE_BROADCAST, 8, (3 * R - 2) * N),
                                   ("reduce", r2.PHASE_REDUCE, 8, (3 * R - 1) * N),
                                   ("all-to-all", r2.PHASE_ALLTOALL, 1, (4 * R - 2) * N)):
        desc = r2.SimDesc(R, S, C, w.align, N, r2.BF16, phases, 0, r2.SCHED_STEPS)
        ws = torch.empty(r2.r2_sim_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
        if phases == r2.PHASE_SENDRECV:
            s = _time_calls(torch, lambda: r2.r2_sendrecv_sim(desc, bufs, recv, epochs, ws))
        elif phases == r2.PHASE_ALLTOALL:
            s = _time_calls(torch, lambda: r2.r2_alltoall_sim(desc, bufs, recv, epochs, ws))
        else:
            s = _time_calls(torch, lambda: r2.r2_collective_sim(desc, bufs, epochs, ws))
        alg = units * e
        print(f"{name:14s} cfg2 shape, channel 2 down: {s * 1e6:10.1f} us/op  {alg / s / 1e9:9.1f} GB/s  "
              f"{100 * alg / s / 1e9 / HBM_PEAK_GBPS:6.2f} % of HBM peak ({alg} algorithmic bytes)", file=out, flush=True)
        del ws
    del recv
    rails_lines(r2, torch, np, wl, out, bufs)


def rails_lines(r2, torch, np, wl, out=sys.stderr, bufs=None):
    """Sec. 6 on top of Sec. 5.1: every server has lost a different rail; a link uses what both of its
    ends still have (per-link tables).  The all-reduce on the cfg2 shape and at the sizes of cfg5."""
    w = wl.cfg2()
    R, N, C, e = w.R, w.N, w.C, 2
    if bufs is None:
        bufs = [_to_device(torch, np, x) for x in wl.make_inputs(w)]
    masks = [0b00000001, 0b00000010, 0, 0, 0b00000100, 0, 0, 0b00001000]
    desc = r2.SimDesc(R, 1, C, w.align, N, r2.BF16, r2.PHASE_AR | r2.PHASE_LINKS, 0, r2.SCHED_STEPS)
    ws = torch.empty(r2.r2_sim_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    call = r2.RailsCall(desc, bufs, r2.static_rails([50000] * C, masks), ws)  # arguments marshalled once
    s = _time_calls(torch, call.run)
    alg = (7 * R - 6) * N * e
    print(f"{'all-reduce':14s} cfg2 shape, four ranks lost a rail each (per-link tables): {s * 1e6:10.1f} us/op  "
          f"{alg / s / 1e9:9.1f} GB/s  {100 * alg / s / 1e9 / HBM_PEAK_GBPS:6.2f} % of HBM peak ({alg} algorithmic bytes)",
          file=out, flush=True)
    del ws, call
    # ... and at the inference sizes of cfg5 (hidden 8192 x tokens), where fused columns take over
    for tokens in (1, 16, 64, 256):
        n = 8192 * tokens
        small = [b[:n] for b in bufs]
        line = []
        for sched in (r2.SCHED_AUTO, r2.SCHED_STEPS):
            desc = r2.SimDesc(R, 1, C, w.align, n, r2.BF16, r2.PHASE_AR | r2.PHASE_LINKS, 0, sched)
            ws = torch.empty(r2.r2_sim_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
            call = r2.RailsCall(desc, small, r2.static_rails([50000] * C, masks), ws)
            line.append(_time_calls(torch, call.run, n=200, warm=20) * 1e6)
            del ws, call
        print(f"{'all-reduce':14s} hidden 8192 x {tokens:3d} tokens, per-link tables: {line[0]:8.1f} us/op as scheduled, "
              f"{line[1]:8.1f} us/op with one launch per step", file=out, flush=True)


def allreduce_size_sweep(r2, torch, np, wl, out=sys.stderr):
    """Message-size sweep of the whole all-reduce in the manner of the paper's microbenchmarks (Sec. 8,
    "AllReduce performance": a sweep over message sizes, without and with failures): 8 ranks, bf16,
    8 channels, 8 KiB ... 128 MiB per rank; no channel down, one down, two down from the start.  The
    schedule is the library's choice.  Rates are algorithmic bytes over time; those of fused runs are
    served by cache ("effective").  A failure must not change the time: the same bytes move, cut
    differently."""
    R, C = 8, 8
    weights = [50000] * C
    print("all-reduce size sweep (8 ranks, bf16): us per op with 0 / 1 / 2 channels down", file=out)
    print(f"{'bytes/rank':>12s} {'schedule':>8s} {'none down':>11s} {'ch 2 down':>11s} {'ch 2,5 down':>12s} {'GB/s (none)':>12s}", file=out)
    g = torch.Generator(device="cpu").manual_seed(7)
    size = 8 << 10
    while size <= 128 << 20:
        N = size // 2
        bufs = [torch.randn(N, generator=g).mul_(0.02).to(torch.bfloat16).cuda() for _ in range(R)]
        desc = r2.SimDesc(R, 1, C, 256, N, r2.BF16, r2.PHASE_AR)
        ws = torch.empty(r2.r2_sim_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
        times = []
        for mask in (0, 0b00000100, 0b00100100):
            call = r2.SimCall(desc, bufs, [(0, mask, weights)], ws)
            n = 2000 if size <= (4 << 20) else 50
            times.append(_time_calls(torch, call.run, n=n, warm=5))
        fused = r2.r2_sim_resolve_schedule(desc, [(0, 0, weights)]) == r2.SCHED_FUSED
        alg = (7 * R - 6) * N * 2
        print(f"{size:12d} {'fused' if fused else 'steps':>8s} {times[0] * 1e6:11.1f} {times[1] * 1e6:11.1f} {times[2] * 1e6:12.1f} "
              f"{alg / times[0] / 1e9:12.1f}", file=out, flush=True)
        del ws, bufs
        torch.cuda.empty_cache()
        size *= 4


def recursive_line(r2, torch, np, wl, out=sys.stderr):
    """Recursive R2CCL-AllReduce (Sec. 6) on the cfg2 shape: rank 0 has lost four of eight NICs, rank 3
    two, rank 5 one; shares from the planner."""
    w = wl.cfg2()
    R, C, e = w.R, w.C, 2
    weights = [50000] * C
    masks = [0b00001111, 0, 0, 0b00000011, 0, 0b00000001, 0, 0]
    levels = r2.r2_recursive_plan(weights, masks)
    total = w.N
    desc = r2.RecursiveDesc(R, C, w.align, total, r2.BF16, len(levels))
    elems = r2.r2_recursive_segments(desc, levels)  # the shares, rounded to what every ring divides into
    xs = wl.make_inputs(w)
    bufs = [_to_device(torch, np, x[:total].copy()) for x in xs]
    ws = torch.empty(r2.r2_recursive_workspace_bytes(desc, levels, elems), dtype=torch.uint8, device="cuda")
    s = _time_calls(torch, lambda: r2.r2_recursive_allreduce_sim(desc, bufs, weights, masks, levels, elems, ws))
    alg = 0
    for l, n in zip(levels, elems):
        p = len(l.ranks())
        m = R - p
        # ring over the p members: 7p-6 units; chain: the m excluded ranks add up (2, then 4 each), the p
        # members add and relay (4 each), the excluded ranks copy and pass on (3 each, the last 2)
        chain = (2 + 4 * (m - 1) + 4 * p + 3 * (m - 1) + 2) if m else 0
        alg += ((7 * p - 6) + chain) * n * e
    depth, times = r2.r2_select_strategy(weights, masks, 1, total * e, 5e-6, 1e3)
    print(f"recursive    {len(levels)} levels, elements {elems}: {s * 1e6:10.1f} us/op  {alg / s / 1e9:9.1f} GB/s  "
          f"{100 * alg / s / 1e9 / HBM_PEAK_GBPS:6.2f} % of HBM peak ({alg} algorithmic bytes); "
          f"selector (alpha 5 us, 50 MB/s per unit of weight) picks depth {depth}", file=out, flush=True)


def warm_reduce_copy_lines(r2, torch, out=sys.stderr):
    """The product's stand-alone r2_reduce_copy (tables, checks and all; one chunk, eight long slices) run
    in the ring step's pattern: call i reads the stage call i-1 wrote and a cold local chunk.  To be read
    beside the bare ring-pattern kernel of stream_mix_lines and the ring step's own launches."""
    C, align = 8, 256
    print("stand-alone r2_reduce_copy (bf16) in the ring step's pattern, us per call:", file=out)
    for mib in (64, 128):
        nbytes = mib << 20
        off = r2.r2_partition([50000] * C, 0b100100, nbytes, align)
        cap = (max(off[c + 1] - off[c] for c in range(C)) + 255) // 256 * 256
        d_off = torch.tensor(off, dtype=torch.int64, device="cuda")

        def filled(n):
            t = torch.empty(n, dtype=torch.uint8, device="cuda")
            t.view(torch.bfloat16).normal_(0.0, 0.02)
            return t

        n_loc = 3072 // mib
        locs = [filled(nbytes) for _ in range(n_loc)]
        st = [[filled(cap) for _ in range(C)] for _ in range(2)]
        cells = []
        for name, op, has_in, has_out in (("sum", r2.OP_SUM, True, True), ("copy, staged", r2.OP_COPY, True, True),
                                          ("last copy", r2.OP_COPY, True, False), ("send", r2.OP_SUM, False, True)):
            calls = [r2.ReduceCopyCall(locs[i % n_loc], r2.BF16, op, st[(i + 1) & 1] if has_in else None,
                                       d_off if has_in else None, st[i & 1] if has_out else None,
                                       d_off if has_out else None, C, cap, nbytes=nbytes) for i in range(2 * n_loc)]
            for i in range(6):
                calls[i % len(calls)].run()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(60):
                calls[i % len(calls)].run()
            e1.record()
            torch.cuda.synchronize()
            cells.append(f"{name} {e0.elapsed_time(e1) / 60 * 1e3:6.1f}")
            del calls
        print(f"  {mib:4d} MiB per stream, channels 2 and 5 down: " + " | ".join(cells), file=out, flush=True)
        del locs, st
        torch.cuda.empty_cache()


def data_values_lines(r2, torch, np, wl, out=sys.stderr):
    """The same cfg2 run on buffers of other contents: this GPU's cache hierarchy moves all-zero lines
    faster than any other data, so a figure measured on zero-filled buffers is not a figure."""
    w = _workload("cfg2")
    print("cfg2 whole run by what the rank buffers hold (same kernels, same bytes), ms per all-reduce:", file=out)
    for name in ("N(0, 0.02) (the workload)", "all zero", "all 1.0"):
        if name.startswith("N("):
            xs = wl.make_inputs(w)
        else:
            one = np.uint16(0x3F80) if name == "all 1.0" else np.uint16(0)
            xs = [np.full(w.N, one, dtype=np.uint16) for _ in range(w.R)]
        run = Runner(r2, torch, np, w, xs)
        ms = run.time_steps(20, 3) / 20 * 1e3
        print(f"  {name:26s} {ms:7.4f} ms  {w.algorithmic_bytes / ms / 1e6 / HBM_PEAK_GBPS:.3f} of the HBM peak", file=out, flush=True)
        del run, xs
        torch.cuda.empty_cache()


def stream_mix_lines(torch, out=sys.stderr):
    """What this GPU's memory system gives bare kernels with the step kernel's access shape and none of its
    tables or slices (csrc/stream_probe.hip, a library of its own): cold mixes of one or two read and write
    streams of 256 MiB each over 3 GiB of rotated buffers, and the ring step's own pattern, in which the
    stage one launch writes is what the next reads, at 64 and 128 MiB per stream (cfg4's and cfg2's launch
    sizes).  The product's launches are to be read against these, not against the nominal peak alone."""
    import ctypes

    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2512_25059_amd", "libr2probe.so")
    if not os.path.exists(path):
        raise RuntimeError("libr2probe.so is not built: run `python -m paper_2512_25059_amd.build` first")
    lib = ctypes.CDLL(path)
    lib.r2probe_cold_mix.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_uint64), ctypes.c_int,
                                     ctypes.c_uint64, ctypes.c_int, ctypes.c_void_p]
    lib.r2probe_ring_pattern.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_uint64), ctypes.c_int, ctypes.c_uint64,
                                         ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int, ctypes.c_void_p]
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)

    def filled(n):  # not zeros: all-zero lines move faster through this GPU's caches than any other data
        t = torch.empty(n, dtype=torch.uint8, device="cuda")
        t.view(torch.bfloat16).normal_(0.0, 0.02)
        return t

    def timed(launch, reps, warm):
        assert launch(warm) == 0
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        assert launch(reps) == 0
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3  # us per launch

    nbytes = 256 << 20
    bufs = [filled(nbytes) for _ in range(12)]
    addrs = (ctypes.c_uint64 * 12)(*[b.data_ptr() for b in bufs])
    print(f"cold stream mixes, {nbytes >> 20} MiB per stream, 12 buffers in rotation, non-temporal accesses "
          "(bare kernel, no tables):", file=out)
    for nr, nw in ((1, 0), (2, 0), (0, 1), (0, 2), (1, 1), (2, 1), (1, 2), (2, 2)):
        us = timed(lambda n: lib.r2probe_cold_mix(nr, nw, addrs, 12, nbytes, n, stream), 40, 4)
        rate = (nr + nw) * nbytes / us / 1e3
        print(f"  {nr}R{nw}W  {us:8.1f} us per launch  {rate:8.1f} GB/s  {rate / HBM_PEAK_GBPS:.3f} of the HBM peak", file=out, flush=True)
    del bufs
    torch.cuda.empty_cache()

    print("the ring step's pattern (locals cold and non-temporal, the stage written cacheable by one launch and read "
          "by the next), bare kernel, us per launch:", file=out)
    streams = {0: 4, 1: 3, 2: 2, 3: 2}
    for mib in (64, 128):
        nbytes = mib << 20
        locs = [filled(nbytes) for _ in range(3072 // mib)]
        laddrs = (ctypes.c_uint64 * len(locs))(*[b.data_ptr() for b in locs])
        sa, sb = filled(nbytes), filled(nbytes)
        cells = []
        for kind, name in ((0, "sum"), (1, "copy, staged"), (2, "last copy"), (3, "send")):
            us = timed(lambda n: lib.r2probe_ring_pattern(kind, laddrs, len(locs), sa.data_ptr(), sb.data_ptr(), nbytes, n, stream), 60, 6)
            cells.append(f"{name} {us:6.1f} ({streams[kind] * nbytes / us / 1e3 / HBM_PEAK_GBPS:.3f})")
        print(f"  {mib:4d} MiB per stream: " + " | ".join(cells), file=out, flush=True)
        del locs, sa, sb
        torch.cuda.empty_cache()


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200,
                    help="timed steps (default: 0.2 s of cfg2, so that one stall of the host or the box weighs little)")
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="cfg2", help="cfg1..cfg4 or cfg5_tok{1,16,64,256}")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--kernel-reps", type=int, default=5)
    ap.add_argument("--schedule", choices=["auto", "steps", "fused", "overlap"], default="auto")
    ap.add_argument("--stage-window-mib", type=float, default=0.0,
                    help="stage bytes one launch may write (0 = library default)")
    ap.add_argument("--headline-only", action="store_true",
                    help="time the named configuration only (no cold figures, no other configurations): for profiler runs")
    ap.add_argument("--all", action="store_true", help="also print a table of every configuration to stderr")
    ap.add_argument("--rails", action="store_true",
                    help="also print the all-reduce with per-link tables (cfg2 shape and cfg5's sizes) to stderr")
    ap.add_argument("--sweep", action="store_true",
                    help="also print size sweeps to stderr: r2_reduce_copy, and the whole all-reduce without and with failures")
    ap.add_argument("--stream-mix", action="store_true",
                    help="also print to stderr what bare kernels with the step kernel's access shape reach on this GPU "
                         "(cold mixes of read and write streams; the ring step's warm pattern), the stand-alone "
                         "r2_reduce_copy in that pattern, and cfg2 on buffers of other contents (zeros move faster)")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (R simulated ranks share its HBM); --gpus must be 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2512_25059_amd as r2
    import workloads as wl

    r2.load_library()  # no fallback: fails loudly if the HIP library is not built
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    w = _workload(args.config)
    xs = wl.make_inputs(w)
    run = Runner(r2, torch, np, w, xs, int(args.stage_window_mib * (1 << 20)),
                 {"auto": 0, "steps": 1, "fused": 2, "overlap": 3}[args.schedule])

    # one pass from pristine inputs, kept for the correctness check
    run.step()
    torch.cuda.synchronize()
    first_pass = [b.cpu().numpy().view(x.dtype) for b, x in zip(run.bufs, xs)]

    secs = run.time_steps(args.steps, args.warmup)
    ms_per_step = secs / args.steps * 1e3
    gbps = w.algorithmic_bytes / (secs / args.steps) / 1e9

    # the same steps one by one, each between a pair of events on the stream they run on: the median
    # says how much a slow outlier weighs in the figure above (launch-bound workloads: the events'
    # own cost shows)
    singles = []
    for _ in range(min(max(args.steps, 1), 50) if not run.fused else 0):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        run.step()
        e1.record()
        torch.cuda.synchronize()
        singles.append(e0.elapsed_time(e1))
    median_ms = sorted(singles)[len(singles) // 2] if singles else None

    # dominant kernel: the fused reducing step that also stages (two reads, two writes per element)
    if run.fused:
        ktimes = run.kernel_times(args.kernel_reps)
        dom = "fused"
        dom_avg_ms, dom_launches = ktimes[dom]
        launch_bytes = w.algorithmic_bytes / len(_fused_segments(w))
        kernel_name = "ring_fused_partition_kernel<%s> (ring_fused_kernel when the tables are prepared up front)" % w.dtype
        served_by = "cache: the stage round trip of a fused column stays in L2 (effective rate, not an HBM figure)"
    else:
        dom, dom_avg_ms, dom_launches, launch_bytes, ktimes = _dominant(run, w, args.kernel_reps)
        kernel_name = {"sum": "ring_step_kernel<Sum%s, staged>" % ("BF16" if w.dtype == "bf16" else "F32"),
                       "copy": "ring_step_kernel<Copy, staged>"}[dom]
        # what one step stages (N*e bytes over all ranks, per pass) is read back by the next launch
        staged = w.N * w.elem_bytes / run.P
        served_by = ("HBM for three of the four streams + Infinity Cache for the incoming stage (the %d MiB a step "
                     "stages are still in the 256 MiB cache when the next launch reads them); frac_cold is the "
                     "all-HBM figure" % (staged // (1 << 20)) if staged <= (128 << 20) else "HBM")
    achieved = launch_bytes / (dom_avg_ms * 1e-3) / 1e9
    traffic, traffic_source = MEASURED_TRAFFIC.get((w.name, dom), (None, None))

    out = {
        "metric": "reduce-copy effective HBM GB/s",
        "value": round(gbps, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_median_of_single_steps": None if median_ms is None else round(median_ms, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {
            "workload": f"{w.name}: R={w.R} ranks, {w.dtype}, {w.N} elems/rank, S={w.S}, C={w.C}, {w.phases}; {w.note}"[:127],
            "algorithmic_bytes_per_step": w.algorithmic_bytes,
            "schedule": "fused columns" if run.fused else "one launch per ring step",
            "passes": run.P,
            # fused runs partition inside their kernels (the epoch lists of these workloads fit the
            # argument block); the step schedule has one partition launch in front
            "launches_per_step": len(_fused_segments(w)) if run.fused else run.P * run.J + 1,
        },
        "pct_of_hbm_peak": round(100.0 * gbps / HBM_PEAK_GBPS, 2),
        "roofline": {
            "bound": "hbm",
            "kernel": kernel_name,
            "achieved": round(achieved, 2),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "served_by": served_by,
            "traffic": traffic,
            "traffic_source": None if traffic is None else
                              f"{traffic_source} (an earlier rocprofv3 --pmc run of this command; not measured by this run)",
            "bytes_per_launch": launch_bytes,
            "avg_launch_ms": round(dom_avg_ms, 5),
            "launches_timed": dom_launches,
        },
        "launch_ms_by_kind": {k: round(v[0], 5) for k, v in ktimes.items()},
        "context": "paper reports <1% training and <3% inference failover overhead on 2x8 H100 InfiniBand "
                   "servers; it gives no kernel-level number, so vs_baseline is null",
    }

    check = not args.no_cpu_baseline
    if check:
        base, ok = _cpu_baseline(w, xs, first_pass, np)
        out["cpu_baseline"] = base
        out["matches_oracle"] = bool(ok)
    del run, xs, first_pass
    torch.cuda.empty_cache()

    if args.config == "cfg2" and not args.headline_only:
        # The other configurations, each in the schedule the library picks for it; and the same chunk
        # worker with every stream coming from and going to HBM (cfg3 once more, in one pass).
        out["configs"] = {}
        for name in OTHER_CONFIGS:
            out["configs"][name], cold = config_entry(r2, torch, np, wl, name, check, args.kernel_reps,
                                                      cold_window=(256 << 20) if name == "cfg3" else 0)
            if cold:
                c3_ms, c3_bytes = cold
            print(f"bench.py: {name} done", file=sys.stderr, flush=True)
        rc_ms, rc_bytes = cold_reduce_copy(r2, torch, "bf16", 256)
        rc_frac = rc_bytes / (rc_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS
        c3_frac = c3_bytes / (c3_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS
        out["roofline"]["frac_cold"] = round(min(rc_frac, c3_frac), 4)
        out["roofline"]["plain_copy_frac"] = round(plain_copy_rate(torch), 4)  # context: a 1 GiB device copy, same units
        out["roofline"]["cold"] = {
            "reduce_copy_bf16_sum_256MiB_chunks_rotated_over_4_buffer_sets": {"avg_launch_ms": round(rc_ms, 5), "frac": round(rc_frac, 4)},
            "cfg3_forced_to_one_pass_f32_sum_1GiB_per_launch": {"avg_launch_ms": round(c3_ms, 5), "frac": round(c3_frac, 4)},
        }
        # the large configurations' dominant-kernel fractions also where the roofline object is read
        out["roofline"]["other_configs"] = {n: {k: out["configs"][n][k] for k in ("kernel", "avg_launch_ms", "frac", "passes")}
                                            for n in ("cfg3", "cfg4")}
        if check:
            out["matches_oracle_all"] = bool(out["matches_oracle"] and all(c["matches_oracle"] for c in out["configs"].values()))

    print(json.dumps(out), flush=True)
    if check and not out.get("matches_oracle_all", out["matches_oracle"]):
        print("bench.py: a GPU result differs from the oracle", file=sys.stderr)
        return 1

    if args.all:
        print("every configuration, schedule chosen by the library (fused columns for launch-bound sizes):", file=sys.stderr)
        for name in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5_tok1", "cfg5_tok16", "cfg5_tok64", "cfg5_tok256"):
            wk = _workload(name)
            rk = Runner(r2, torch, np, wk, wl.make_inputs(wk))
            n = 10000 if name.startswith("cfg5") else (2000 if name == "cfg1" else 20)
            s = rk.time_steps(n, 3) / n
            rate = wk.algorithmic_bytes / s / 1e9
            # a fused run's stage traffic never leaves the caches: its rate is not an HBM figure
            tail = "effective (cache-served)" if rk.fused else f"{100 * rate / HBM_PEAK_GBPS:6.2f} % of HBM peak"
            line = (f"{name:12s} {'fused' if rk.fused else 'steps':5s} {n:6d} back-to-back ops {s * 1e6:10.1f} us/op  "
                    f"{rate:9.1f} GB/s  {tail}")
            if name.startswith("cfg5"):
                # the back-to-back loop runs in place (values grow, then saturate); confirm once with
                # inputs restored before every op that this does not change the timing
                tot = 0.0
                for _ in range(100):
                    rk.restore()
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    rk.step()
                    e1.record()
                    torch.cuda.synchronize()
                    tot += e0.elapsed_time(e1)
                line += f"  | restored inputs, GPU time per op: {tot / 100 * 1e3:.1f} us"
            if rk.fused:
                line += f"  | replayed from a HIP graph of 100 ops: {rk.graph_seconds_per_op() * 1e6:.1f} us/op"
            print(line, file=sys.stderr, flush=True)
            del rk
            torch.cuda.empty_cache()
        split_line(r2, torch, np, wl)
        recursive_line(r2, torch, np, wl)
        other_collectives_lines(r2, torch, np, wl)
    if args.rails and not args.all:
        rails_lines(r2, torch, np, wl)
    if args.stream_mix:
        stream_mix_lines(torch)
        warm_reduce_copy_lines(r2, torch)
        data_values_lines(r2, torch, np, wl)
    if args.sweep:
        reduce_copy_sweep(r2, torch)
        allreduce_size_sweep(r2, torch, np, wl)
    return 0


if __name__ == "__main__":
    sys.exit(main())
