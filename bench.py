"""Benchmark of the chunked N-way reduce on one MI355X.

One step = one hop_reduce call over the asynchronous-SGD workload (16 fp32
objects of 64 MiB, the first 12 ready are reduced, 4 MiB chunks, tree degree
4), inputs resident in HBM. Prints ONE JSON line with the metric, the
roofline of the reduce kernel and the CPU oracle's rate on a bounded sample.
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

HBM_PEAK_GBS = 8000.0       # MI355X published peak HBM3E bandwidth, GB/s (1e9 B/s)

# HBM bytes moved by ONE reduce launch of workload 2, from two rocprofv3 --pmc runs (FETCH_SIZE, then
# WRITE_SIZE), each scaled by what the same counter read for the 256 MiB copy probe of this file
# (profiles/reduce_kernel_cfg2_async_sgd.md). Valid only for the kernel launch shape named here: if the
# library reports another one, the figure is withheld (null).
MEASURED_TRAFFIC = {
    "workload": "cfg2_async_sgd",
    "kernel_config": "reduce: 64 lanes/workgroup, 4|2|1 vectors/lane by accumulator depth, unroll 1; below 768 4-KiB "
                     "tiles: 1 KiB tiles, unroll 8; below 2048: 2 KiB per workgroup, unroll 2, in two pieces 16 KiB apart;"
                     " from 2048: 1 KiB pieces 64 KiB apart, one per vector (the 2 KiB shape instead if the rounds of "
                     "resident waves would be less than 80 % full); kernels with 4 vectors/lane: 8 waves per CU from 5120 "
                     "tiles; bf16 at depth 5..8 from 768 tiles: 2 vectors/lane, unroll 2 (pieces 64 KiB apart from 2048 "
                     "tiles); groups of 8 plain steps marked by the host; nontemporal loads+stores, programs <= 128 steps "
                     "in kernel arguments; vector grids start at a 128-byte boundary of the sources (reduce) or "
                     "destinations (copies); copy to one destination: 64 lanes/workgroup, 8 contiguous vectors/lane; from "
                     "5120 8-KiB tiles 4 vectors/lane in 1 KiB pieces 64 KiB apart, 10 waves per CU; nontemporal; to "
                     "several: one 4 KiB tile and one destination per workgroup, destination-major within spans of 4096 "
                     "tiles, cached loads, nontemporal stores, 12 waves per CU (no limit for >= 128 MiB to < 8 "
                     "destinations)",
    "bytes": 872313828,
}


def time_calls(fn, steps, warmup, torch):
    """Average device time per call in ms, bracketed by events on the current stream."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return e0.elapsed_time(e1) / steps, wall_ms / steps


def time_calls_median(fn, steps, warmup, torch, batch=100):
    """For launch-bound workloads: the timed calls are taken in batches and the median batch is
    reported, so that a one-off stall of the runtime (tens of ms, a few times per process, at launch
    counts that depend on nothing the library does) does not decide the figure."""
    import statistics
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    dev_ms, wall_ms = [], []
    for _ in range(max(1, steps // batch)):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(batch):
            fn()
        e1.record()
        torch.cuda.synchronize()
        wall_ms.append((time.perf_counter() - t0) * 1e3 / batch)
        dev_ms.append(e0.elapsed_time(e1) / batch)
    return statistics.median(dev_ms), statistics.median(wall_ms)


def cpu_baseline(w, objs, order, torch, sample_elems, min_seconds=10.0):
    """The oracle as it stands, single thread, on the first sample_elems elements of every object, repeated
    until about min_seconds of CPU time have been spent; the mean rate is reported."""
    import numpy as np

    import oracle
    import workloads
    host = [workloads.to_numpy(o[:sample_elems]) for o in objs]
    reps, spent, out, k_eff = 0, 0.0, None, 0
    while reps < 2 or spent < min_seconds:
        t0 = time.perf_counter()
        rc, out, k_eff, _ = oracle.reduce(host, w.k, oracle.SUM, oracle.F32, w.chunk_bytes // 4, w.tree_degree, order,
                                          None)
        spent += time.perf_counter() - t0
        reps += 1
    nbytes = (k_eff + 1) * sample_elems * 4
    return {"value": round(nbytes * reps / spent / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": "%d passes over the first %d of %d elements of each object (%.0f MB counted per pass), %.1f s" %
                      (reps, sample_elems, w.n_elems, nbytes / 1e6, spent)}, out


def paced_arrivals(hop, torch, w, objs, order, dst, interval_us, reps=5):
    """Objects become ready whole, one every interval_us (host clock), in the workload's ready order; only
    the first k matter. Measured: host time from the last arrival to the completed result (stream
    synchronised), median of reps, for the fused policy (one launch when everything is there), the
    eager one (every arrival folded into saved accumulators at once) and the adaptive one (eager, but only
    while the stream has nothing left to do)."""
    import statistics
    table = hop.PtrTable(objs)
    C = w.n_chunks
    res = {"interval_us": interval_us, "k": w.k}
    for name, eager in (("fused", 0), ("eager", 1), ("adaptive", 1)):
        tails, launches = [], 0
        for _ in range(reps + 1):
            rc, s = hop.hop_session_begin(dst, table, w.k, w.ops[0], w.dtype, w.chunk_bytes, w.tree_degree)
            assert rc == hop.HOP_OK, hop.hop_strerror(rc)
            hop.hop_session_set_eager(s, eager)
            hop.hop_session_set_adaptive(s, name == "adaptive")
            torch.cuda.synchronize()
            t_next = time.perf_counter()
            for t in range(w.k):
                while time.perf_counter() < t_next:
                    pass
                t_last = time.perf_counter()
                assert hop.hop_session_ready(s, int(order[t]), C) == hop.HOP_OK
                t_next += interval_us * 1e-6
            rc, info = hop.hop_session_finish(s)
            torch.cuda.synchronize()
            tails.append((time.perf_counter() - t_last) * 1e6)
            launches = info["n_launches"]
            assert rc == hop.HOP_OK
        res[name] = {"us_after_last_arrival": round(statistics.median(tails[1:]), 1), "launches": launches}
    return res


def streamed_chunks(hop, torch, w, objs, order, dst, interval_us, reps=5):
    """All k objects stream side by side: every interval_us (host clock) each of them has one more chunk.
    Measured: host time from the last notification to the completed result, and the launches it took, with
    the default policy (a launch per chunk run as soon as all k have it): the pipelining of section 3.3."""
    import statistics
    table = hop.PtrTable(objs)
    C = w.n_chunks
    first_k = [int(order[t]) for t in range(w.k)]
    res = {"interval_us": interval_us, "k": w.k, "chunks": C}
    for name in ("fused",):
        tails, totals, launches = [], [], 0
        for _ in range(reps + 1):
            rc, s = hop.hop_session_begin(dst, table, w.k, w.ops[0], w.dtype, w.chunk_bytes, w.tree_degree)
            assert rc == hop.HOP_OK, hop.hop_strerror(rc)
            for i in first_k:
                assert hop.hop_session_ready(s, i, 0) == hop.HOP_OK
            torch.cuda.synchronize()
            t_begin = t_next = time.perf_counter()
            for c in range(1, C + 1):
                while time.perf_counter() < t_next:
                    pass
                for i in first_k:
                    assert hop.hop_session_ready(s, i, c) == hop.HOP_OK
                t_last = time.perf_counter()
                t_next += interval_us * 1e-6
            rc, info = hop.hop_session_finish(s)
            torch.cuda.synchronize()
            t_end = time.perf_counter()
            tails.append((t_end - t_last) * 1e6)
            totals.append((t_end - t_begin) * 1e6)
            launches = info["n_launches"]
            assert rc == hop.HOP_OK
        res[name] = {"us_after_last_chunk": round(statistics.median(tails[1:]), 1),
                     "us_first_chunk_to_result": round(statistics.median(totals[1:]), 1), "launches": launches}
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50,
                    help="untimed calls before the timed ones (the first few dozen calls of a process run at lower clocks)")
    ap.add_argument("--workload", type=int, default=2, help="which of the five workloads (default: 2)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--all-configs", action="store_true", help="also time the other workloads (extra JSON field)")
    ap.add_argument("--streamed-interval-us", type=float, default=None,
                    help="also: all k objects stream chunk by chunk, one more chunk each per interval")
    ap.add_argument("--paced-interval-us", type=float, default=None,
                    help="also run the workload's objects through the event-level API, one whole object every "
                         "INTERVAL microseconds, and report how long after the last arrival the result is complete, "
                         "for the fused and the eager scheduling policy (the paper's asynchrony experiment)")
    ap.add_argument("--degree-sweep", action="store_true",
                    help="also time the workload with tree degrees 1, 2, 4, 8 and k (the ablation of the paper's "
                         "appendix B, on one GPU: the degree fixes the association order and the accumulator depth, "
                         "not the traffic)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run hop_broadcast of one 256 MiB object to one destination a few times: a copy of "
                         "known size against which hardware byte counters can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs one node's share of the reduce on ONE GPU; --gpus %d is not supported "
              "(no collectives between GPUs exist in it)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2002_05814_amd as hop
    import workloads

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    hop.lib()                                   # fails loudly if the HIP library is not built
    dev = torch.device("cuda:0")

    def run_workload(cfg, steps, warmup, no_fail=False, timer=time_calls):
        w = workloads.WORKLOADS[cfg]
        if no_fail:
            w = w.scaled(w.object_bytes, fail={}, name=w.name + "_without_failure")
        objs = workloads.make_objects(w, device=dev)
        order, fm = w.ready_order(), w.fail_mask()
        n_out = max(1, w.n_dst)
        # two destination sets, alternated, so that a call never finds its output lines in cache
        dsts = [[torch.empty_like(objs[0]) for _ in range(n_out)] for _ in range(2)]
        # Workloads whose inputs would all sit in the 256 MB last-level cache get 64 copies of the input
        # set at different addresses (>= 256 MiB in total), used in turn.
        total = w.n * w.object_bytes
        n_sets = 1 if total > (64 << 20) else max(64, -(-(256 << 20) // total))
        obj_sets = [objs]
        for _ in range(n_sets - 1):
            block = torch.stack(objs)                      # one allocation, objects object_bytes apart
            obj_sets.append([block[i] for i in range(w.n)])
        # pointer tables are marshalled once, as a caller that reuses its buffers would
        obj_tables = [hop.PtrTable(o) for o in obj_sets]
        dst_tables = [hop.PtrTable(d) for d in dsts]
        results = {}
        for op in w.ops:
            state = {"i": 0, "info": None, "rc": 0}

            def step():
                d = dsts[state["i"] & 1]
                obj_table = obj_tables[state["i"] % n_sets]
                state["i"] += 1
                if w.n_dst:
                    state["rc"], state["info"] = hop.hop_allreduce(dst_tables[(state["i"] - 1) & 1], obj_table, w.k,
                                                                   op, w.dtype, w.chunk_bytes, w.tree_degree,
                                                                   order, fm)
                else:
                    state["rc"], state["info"] = hop.hop_reduce(d[0], obj_table, w.k, op, w.dtype, w.chunk_bytes,
                                                                w.tree_degree, order, fm)
            ms, wall_ms = timer(step, steps, warmup, torch)
            assert state["rc"] >= 0, hop.hop_strerror(state["rc"])
            k_eff = state["info"]["k_eff"]
            counted = (k_eff + 1) * w.object_bytes
            if w.n_dst:
                counted = (k_eff + w.n_dst) * w.object_bytes        # least traffic of reduce + broadcast
            # what the launches really moved (repairs included), from the scheduler's own account
            moved = (state["info"]["chunk_steps"] + state["info"]["chunk_stores"]) * min(w.chunk_bytes, w.object_bytes)
            if w.n_dst:
                moved += w.n_dst * w.object_bytes       # copy kernel: 1 read + (n_dst - 1) writes
            results[op] = {"ms": ms, "wall_ms": wall_ms, "gbs": counted / (ms * 1e-3) / 1e9, "bytes": counted,
                           "moved_gbs": moved / (ms * 1e-3) / 1e9, "info": state["info"], "status": state["rc"]}
        return w, objs, order, dsts, results

    w, objs, order, dsts, res = run_workload(args.workload, args.steps, args.warmup)
    op = w.ops[0]
    r = res[op]
    out = {
        "metric": "reduce input GB/s and % of MI355X HBM peak, N-way chunked reduce",
        "value": round(r["gbs"], 2),
        "unit": "GB/s",
        "pct_of_hbm_peak": round(100.0 * r["gbs"] / HBM_PEAK_GBS, 2),
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(r["ms"], 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": {"f32": "f32", "bf16": "bf16 in, f32 accumulate", "i32": "int32"}[w.dtype],
        "data": "synthetic",
        "config": {"workload": w.name, "n": w.n, "k": w.k, "object_bytes": w.object_bytes,
                   "chunk_bytes": w.chunk_bytes, "tree_degree": r["info"]["degree_used"], "op": op,
                   "counted_bytes": r["bytes"], "launches_per_step": r["info"]["n_launches"],
                   "host_ms_per_step": round(r["wall_ms"], 5)},
        "roofline": {"bound": "hbm", "achieved": round(r["gbs"], 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(r["gbs"] / HBM_PEAK_GBS, 4),
                     "traffic": (MEASURED_TRAFFIC["bytes"]
                                 if (w.name == MEASURED_TRAFFIC["workload"]
                                     and hop.hop_kernel_config() == MEASURED_TRAFFIC["kernel_config"]) else None),
                     "kernel": "hop::reduce_kernel", "per_unit": "(k_eff+1) x object_bytes per launch"},
    }
    if not args.no_cpu_baseline and w.dtype == "f32" and not w.n_dst:
        sample = w.n_elems                      # the whole workload; repeated to about 10 s of CPU time
        base, want = cpu_baseline(w, objs, order, torch, sample)
        got = workloads.to_numpy(dsts[(args.steps + args.warmup - 1) & 1][0][:sample])
        base["matches_gpu_bits"] = bool(np.array_equal(got.view(np.uint32), want.view(np.uint32)))
        out["cpu_baseline"] = base
    else:
        out["cpu_baseline"] = None
    if args.copy_probe:
        src = torch.ones(64 << 20, dtype=torch.float32, device=dev)
        dstp = torch.empty_like(src)

        def probe():
            assert hop.hop_broadcast([dstp], src, 4 << 20) == hop.HOP_OK
        ms, _ = time_calls(probe, 10, 2, torch)
        out["copy_probe"] = {"bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4, "ms": round(ms, 5),
                             "GB/s_read_plus_write": round(2 * src.numel() * 4 / (ms * 1e-3) / 1e9, 2),
                             "kernel": "hop::copy_kernel"}
        del src, dstp
    if args.degree_sweep:
        sweep = {}
        table = hop.PtrTable(objs)
        for deg in (1, 2, 4, 8, w.k):
            st = {"i": 0, "info": None}

            def step_deg():
                st["i"] += 1
                _, st["info"] = hop.hop_reduce(dsts[st["i"] & 1][0], table, w.k, op, w.dtype, w.chunk_bytes, deg, order,
                                               None)
            ms, _ = time_calls(step_deg, max(20, args.steps // 4), 10, torch)
            nbytes = (st["info"]["k_eff"] + 1) * w.object_bytes        # reduce only, nobody fails
            sweep["d=%d" % deg] = {"ms": round(ms, 5), "GB/s": round(nbytes / (ms * 1e-3) / 1e9, 1),
                                   "levels": st["info"]["stack_depth"]}
        sweep["picked_by_eq1"] = hop.hop_pick_degree(w.k, w.object_bytes, 0.0, 0.0)
        out["degree_sweep"] = sweep
    if args.streamed_interval_us is not None:
        out["streamed_chunks"] = streamed_chunks(hop, torch, w, objs, order, dsts[0][0], args.streamed_interval_us)
    if args.paced_interval_us is not None:
        out["paced_arrivals"] = paced_arrivals(hop, torch, w, objs, order, dsts[0][0], args.paced_interval_us)
    if args.all_configs:
        extra = {}
        del objs, dsts
        torch.cuda.empty_cache()
        for cfg, no_fail in ((1, False), (3, False), (4, False), (4, True), (5, False)):
            # the tiny workloads are launch-bound: median over batches of 100 calls (see time_calls_median)
            tiny = cfg in (1, 5)
            wk, o2, _, d2, rs = run_workload(cfg, 1000 if tiny else max(10, args.steps // 5),
                                             300 if tiny else 20, no_fail, time_calls_median if tiny else time_calls)
            for opn, rr in rs.items():
                extra["%s/%s" % (wk.name, opn)] = {"GB/s": round(rr["gbs"], 2), "ms": round(rr["ms"], 5),
                                                  "frac_of_hbm_peak": round(rr["gbs"] / HBM_PEAK_GBS, 4),
                                                  "counted_bytes": rr["bytes"], "status": rr["status"],
                                                  "GB/s_moved_incl_repair": round(rr["moved_gbs"], 2),
                                                  "launches": rr["info"]["n_launches"]}
            del o2, d2
            torch.cuda.empty_cache()
        out["all_configs"] = extra
    print(json.dumps(out))


if __name__ == "__main__":
    main()
