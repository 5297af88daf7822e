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

# HBM bytes moved per call, from two rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE), each scaled by what
# the same counter read for the 256 MiB copy probe of this file; summed over the call's launches. The
# summaries are in profiles/ (with the commands that made them). The figures hold only for the kernel launch
# shapes they were taken with: they are reported only while the library's hop_kernel_config() string is the
# one recorded here (else null).
PROFILED_TRAFFIC = {
    "kernel_config": (
                     "reduce: 64 lanes/workgroup, 4|2|1 vectors/lane by accumulator depth, unroll 1; below 768 4-KiB "
                     "tiles: 1 KiB tiles, unroll 8; below 2048: 2 KiB per workgroup, unroll 2, in two pieces 16 KiB apart; "
                     "from 2048: 1 KiB pieces 64 KiB apart, one per vector (the 2 KiB shape instead if the rounds of "
                     "resident waves would be less than 80 % full); kernels with 4 vectors/lane: 8 waves per CU from 5120 "
                     "tiles; bf16 at depth 5..8 from 768 tiles: 2 vectors/lane, unroll 2 (pieces 64 KiB apart from 2048 "
                     "tiles); groups of 8 plain steps marked by the host; nontemporal loads+stores, programs <= 128 steps "
                     "in kernel arguments; vector grids start at a 128-byte boundary of the sources (reduce) or "
                     "destinations (copies); copy to one destination: 64 lanes/workgroup, 8 contiguous vectors/lane; from "
                     "5120 8-KiB tiles 4 vectors/lane in 1 KiB pieces 64 KiB apart, 10 waves per CU; nontemporal; to "
                     "several: one 4 KiB tile and one destination per workgroup, destination-major within spans of 4096 "
                     "tiles, cached loads, nontemporal stores, 12 waves per CU (no limit for >= 128 MiB to < 8 "
                     "destinations); launches that keep or read partial results: one step at a time, 4|2|1 vectors/lane, "
                     "pieces 64 KiB apart from 2048 tiles, 8 waves per CU from 5120 tiles, partials as 4-byte accumulators "
                     "indexed like the elements, nontemporal; programs of 48 steps or more over at most 64 KiB: one "
                     "launch, 256 lanes per 64-byte column, chains of at most 23 items folded by teams of 4 lanes with all "
                     "their loads in flight, values in LDS, tables of up to 256 chains in the kernel arguments, "
                     "four columns in a row per die; above 64 KiB up to 768 KiB: 512 lanes per 1 KiB column, a wave per chain"),
    "workloads": {
        "cfg2_async_sgd": {"bytes_per_call": 872327474, "profile": "profiles/hbm_traffic_all_workloads.md"},
        "cfg3_rl_allreduce": {"bytes_per_call": 2163381761, "profile": "profiles/hbm_traffic_all_workloads.md"},
        "cfg4_large_fault": {"bytes_per_call": 10181969677, "profile": "profiles/hbm_traffic_all_workloads.md"},
        "cfg4_large_fault_without_failure": {"bytes_per_call": 8856980408, "profile": "profiles/hbm_traffic_all_workloads.md"},
    },
}

# The paper's own headline results (its sections 5.2-5.4 and 5 "setup"): context, not a target.
PAPER_CONTEXT = {
    "source": "arXiv 2002.05814 (SIGCOMM '21), sections 5.2-5.4",
    "speedups_over_ray": {"async_sgd_parameter_server_16_nodes": "7.8x AlexNet / 7.0x VGG-16 / 5.0x ResNet-50",
                          "rl_16_nodes": "3.9x A3C, 1.8x IMPALA", "ensemble_serving_16_nodes": "3.3x (2.2x on 8 nodes)"},
    "hardware": "AWS EC2, 16 m5.4xlarge nodes (16 vCPUs, 64 GB, 10 Gbps network = 1.25 GB/s per node); the "
                "application runs on 8 or 16 p3.2xlarge nodes (one V100 each, same network); CPU objects only, no GPU "
                "path in the paper",
    "note": "speedups of whole applications over Ray on a 10 Gbps cluster; nothing there is comparable with a "
            "fraction of one GPU's HBM bandwidth",
}


def profiled_traffic(workload_name, kernel_config):
    """Counter-measured HBM bytes per call of this workload ({"bytes_per_call", "profile"}), or None if there
    is no profile for it or the library's launch shapes have changed since the counters were taken."""
    entry = PROFILED_TRAFFIC["workloads"].get(workload_name)
    if not entry or PROFILED_TRAFFIC["kernel_config"] != kernel_config:
        return None
    return entry


def time_calls(fn, steps, warmup, torch):
    """Device time per call in ms over exactly `steps` calls enqueued back to back between two events on the
    current stream (the stream the kernels are launched on): (mean over all calls, host wall mean, median over
    batches). An event behind every call would cost 2-3 us per call (the next kernel no longer starts while
    the previous one drains), so the calls are marked in batches of at least 10 (a tenth of the steps)."""
    import statistics
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    batch = max(10, steps // 10)
    edges = list(range(0, steps, batch)) + [steps]
    marks = [torch.cuda.Event(enable_timing=True) for _ in edges]
    t0 = time.perf_counter()
    marks[0].record()
    nxt = 1
    for i in range(steps):
        fn()
        if i + 1 == edges[nxt]:
            marks[nxt].record()
            nxt += 1
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    each = [marks[j].elapsed_time(marks[j + 1]) / (edges[j + 1] - edges[j]) for j in range(len(edges) - 1)]
    return marks[0].elapsed_time(marks[-1]) / steps, wall_ms / steps, statistics.median(each)


def time_calls_median(fn, steps, warmup, torch, batch=100):
    """For launch-bound workloads (a call takes 10-30 us, an event behind every call would be part of what is
    measured): the timed calls are taken in batches of 100; mean and median over the batches are reported."""
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
    return statistics.mean(dev_ms), statistics.median(wall_ms), statistics.median(dev_ms)


# A caller written in C: the same hop_reduce call in a plain loop, to separate the library's host cost per
# call from the Python binding's. Compiled with gcc when bench.py runs (nothing of the method is in it).
C_LOOP_SOURCE = r"""
#include <stddef.h>
#include <stdint.h>
#include <time.h>
typedef int (*reduce_fn)(void *, const void *const *, int, size_t, const int32_t *, int, int, int, size_t, int,
                         const int64_t *, void *, void *);
double c_loop(reduce_fn f, int repeats, void *const *dsts, int n_dsts, const void *const *const *obj_sets, int n_sets,
              int n, size_t object_bytes, const int32_t *order, int k, int op, int dtype, size_t chunk_bytes, int degree,
              void *stream, int *status)
{
    struct timespec t0, t1;
    clock_gettime(CLOCK_MONOTONIC, &t0);
    for (int i = 0; i < repeats; ++i) {
        int rc = f(dsts[i % n_dsts], obj_sets[i % n_sets], n, object_bytes, order, k, op, dtype, chunk_bytes, degree, 0,
                   stream, 0);
        if (rc < 0) { *status = rc; break; }
    }
    clock_gettime(CLOCK_MONOTONIC, &t1);
    return (t1.tv_sec - t0.tv_sec) + 1e-9 * (t1.tv_nsec - t0.tv_nsec);
}
"""


def c_loop_host_time(hop, torch, w, obj_tables, dsts, order, op, repeats=3000):
    """Host seconds per hop_reduce call from a C loop (the stream is synchronised before and after; the
    loop itself only enqueues), and the device-inclusive time per call of the same loop. None without gcc."""
    import ctypes
    import shutil
    import subprocess
    import tempfile
    if shutil.which("gcc") is None:
        return None
    with tempfile.TemporaryDirectory(prefix="hop_cloop_") as tmp:
        src, lib = os.path.join(tmp, "cloop.c"), os.path.join(tmp, "cloop.so")
        with open(src, "w") as f:
            f.write(C_LOOP_SOURCE)
        subprocess.run(["gcc", "-O2", "-shared", "-fPIC", src, "-o", lib], check=True)
        L = ctypes.CDLL(lib)
        L.c_loop.restype = ctypes.c_double
        n_sets = len(obj_tables)
        sets = (ctypes.c_void_p * n_sets)(*[ctypes.cast(t.array, ctypes.c_void_p) for t in obj_tables])
        dptr = (ctypes.c_void_p * len(dsts))(*[int(d.data_ptr()) for d in dsts])
        oarr = order.astype("int32")
        status = ctypes.c_int(0)
        fn = ctypes.cast(hop.lib().hop_reduce, ctypes.c_void_p)
        stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        args = (fn, repeats, dptr, len(dsts), sets, n_sets, w.n, ctypes.c_size_t(w.object_bytes),
                oarr.ctypes.data_as(ctypes.c_void_p), w.k, hop.OPS[op], hop.DTYPES[w.dtype], ctypes.c_size_t(w.chunk_bytes),
                w.tree_degree, stream, ctypes.byref(status))
        L.c_loop.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_int,
                             ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                             ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        L.c_loop(*args)                                   # warm-up (and records the calls)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        L.c_loop(*args)
        torch.cuda.synchronize()
        total_s = time.perf_counter() - t0
        # the host's share: a burst short enough for the launch queue to take it without pushing back
        burst = 200
        short = list(args)
        short[1] = burst
        host_s = min(L.c_loop(*short) + 0.0 * (torch.cuda.synchronize() or 0) for _ in range(5))
        torch.cuda.synchronize()
        if status.value < 0:
            return None
        return {"host_us_per_call": round(host_s / burst * 1e6, 3), "us_per_call_with_device": round(total_s / repeats * 1e6, 3),
                "calls": repeats, "host_burst": burst}


def host_description():
    """CPU model and core counts of the machine the oracle is timed on."""
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    try:
        usable = len(os.sched_getaffinity(0))
    except (AttributeError, OSError):
        usable = os.cpu_count() or 1
    return {"cpu_model": model, "nproc": os.cpu_count() or 1, "usable_cores": usable}


def cpu_baseline(w, objs, order, torch, sample_elems, min_seconds=10.0, all_core_seconds=4.0, max_threads=16):
    """The oracle as it stands on the first sample_elems elements of every object. Leg 1 (the reported value):
    one thread, repeated until about min_seconds of CPU time have been spent. Leg 2: the same oracle call per
    contiguous slice of elements (the reduce is elementwise, so slices are independent), the slices spread over
    the host's usable cores (at most max_threads) by a thread pool; core count stated."""
    import concurrent.futures

    import numpy as np

    import oracle
    import workloads
    host = [workloads.to_numpy(o[:sample_elems]) for o in objs]
    ce = w.chunk_bytes // 4
    reps, spent, out, k_eff = 0, 0.0, None, 0
    while reps < 2 or spent < min_seconds:
        t0 = time.perf_counter()
        rc, out, k_eff, _ = oracle.reduce(host, w.k, oracle.SUM, oracle.F32, ce, w.tree_degree, order, None)
        spent += time.perf_counter() - t0
        reps += 1
    nbytes = (k_eff + 1) * sample_elems * 4
    desc = host_description()
    base = {"value": round(nbytes * reps / spent / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": "%d passes over the first %d of %d elements of each object (%.0f MB counted per pass), %.1f s" %
                      (reps, sample_elems, w.n_elems, nbytes / 1e6, spent),
            "host": desc}
    # leg 2: all usable cores
    threads = max(1, min(desc["usable_cores"], max_threads))
    cuts = np.linspace(0, sample_elems, 4 * threads + 1).astype(np.int64) // ce * ce
    cuts[-1] = sample_elems
    spans = [(int(a), int(b)) for a, b in zip(cuts[:-1], cuts[1:]) if b > a]

    def one(span):
        a, b = span
        rc2, part, _, _ = oracle.reduce([h[a:b] for h in host], w.k, oracle.SUM, oracle.F32, ce, w.tree_degree, order, None)
        return a, b, part
    reps2, spent2, same = 0, 0.0, True
    with concurrent.futures.ThreadPoolExecutor(max_workers=threads) as pool:
        while reps2 < 1 or spent2 < all_core_seconds:
            t0 = time.perf_counter()
            parts = list(pool.map(one, spans))
            spent2 += time.perf_counter() - t0
            reps2 += 1
        for a, b, part in parts:
            same = same and bool(np.array_equal(part.view(np.uint32), out[a:b].view(np.uint32)))
    base["all_cores"] = {"value": round(nbytes * reps2 / spent2 / 1e9, 4), "unit": "GB/s", "cores": threads,
                         "sample": "%d passes, %d slices per pass, %.1f s" % (reps2, len(spans), spent2),
                         "equals_single_thread_bits": same}
    return base, out


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
    # while the chunks stream in every participant can still fail, so by default each launch also keeps the
    # partial results of subtrees (failure repair); "fused_no_keeping" switches that off
    for name in ("fused", "fused_no_keeping"):
        tails, totals, launches = [], [], 0
        for _ in range(reps + 1):
            rc, s = hop.hop_session_begin(dst, table, w.k, w.ops[0], w.dtype, w.chunk_bytes, w.tree_degree)
            assert rc == hop.HOP_OK, hop.hop_strerror(rc)
            hop.hop_session_set_retention(s, name == "fused")
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
                     "us_first_chunk_to_result": round(statistics.median(totals[1:]), 1), "launches": launches,
                     "partials_kept_per_chunk": info["partial_stores"] // max(1, C)}
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50,
                    help="untimed calls before the timed ones (the first few dozen calls of a process run at lower clocks)")
    ap.add_argument("--workload", type=int, default=2, help="which of the five workloads (default: 2)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--all-configs", action="store_true", help="(default behaviour now; kept for old command lines)")
    ap.add_argument("--skip-all-configs", action="store_true",
                    help="time only the headline workload, not the other four (they take a few seconds)")
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
    ap.add_argument("--size-sweep", action="store_true",
                    help="also time the workload's reduce (same n, k, degree, type) at object sizes from 1 to 64 MiB, "
                         "inputs not cached, and fit time = fixed cost + bytes / rate: what part of a mid-size launch "
                         "is the launch and what part the kernel")
    ap.add_argument("--many-objects-sweep", action="store_true",
                    help="also time sums over 128..4000 inputs of 1 KiB..1 MiB in a 16-ary tree (launch- and "
                         "latency-bound calls: us per call and GB/s per shape)")
    ap.add_argument("--many-objects-dtype", choices=["f32", "bf16", "i32"], default="f32")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run hop_broadcast of one 256 MiB object to one destination a few times: a copy of "
                         "known size against which hardware byte counters can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs one node's share of the reduce on ONE GPU; --gpus %d is not supported "
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
    # CPython's full garbage collection walks every tracked object of the process (170 000 after importing
    # torch: 30-40 ms), and the per-call objects of the binding trigger one every few thousand calls, in the
    # middle of whatever loop is being timed. What exists now is long-lived: it is moved out of the
    # collector's sight, as a serving process would do after start-up.
    import gc
    gc.collect()
    gc.freeze()

    def run_workload(cfg, steps, warmup, no_fail=False, timer=time_calls):
        w = workloads.WORKLOADS[cfg] if cfg in workloads.WORKLOADS else workloads.EXTRA_WORKLOADS[cfg]
        if no_fail:
            w = w.scaled(w.object_bytes, fail={}, name=w.name + "_without_failure")
        objs = workloads.make_objects(w, device=dev)
        order, fm = w.ready_order(), w.fail_mask()
        n_out = max(1, w.n_dst)
        # two destination sets, alternated, so that a call never finds its output lines in cache
        dsts = [[torch.empty_like(objs[0]) for _ in range(n_out)] for _ in range(2)]
        # Workloads whose inputs would all sit in the 256 MB last-level cache get at least 64 copies of the
        # input set at different addresses (>= 512 MiB in total, twice that cache), used in turn.
        total = w.n * w.object_bytes
        n_sets = 1 if total > (64 << 20) else max(64, -(-(512 << 20) // total))
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

            stream = torch.cuda.current_stream().cuda_stream        # looked up once, as a caller in a loop would

            def step():
                d = dsts[state["i"] & 1]
                obj_table = obj_tables[state["i"] % n_sets]
                state["i"] += 1
                if w.n_dst:
                    state["rc"], state["info"] = hop.hop_allreduce(dst_tables[(state["i"] - 1) & 1], obj_table, w.k,
                                                                   op, w.dtype, w.chunk_bytes, w.tree_degree,
                                                                   order, fm, stream=stream)
                else:
                    state["rc"], state["info"] = hop.hop_reduce(d[0], obj_table, w.k, op, w.dtype, w.chunk_bytes,
                                                                w.tree_degree, order, fm, stream=stream)
            ms, wall_ms, ms_median = timer(step, steps, warmup, torch)
            assert state["rc"] >= 0, hop.hop_strerror(state["rc"])
            info = state["info"]
            k_eff = info["k_eff"]
            counted = (k_eff + 1) * w.object_bytes
            if w.n_dst:
                counted = (k_eff + w.n_dst) * w.object_bytes        # least traffic of reduce + broadcast
            # what the launches really moved (repairs and kept partial results included), from the
            # scheduler's own account: source chunks read, result chunks written, partials (4 bytes per element)
            cb = min(w.chunk_bytes, w.object_bytes)
            moved = (info["chunk_steps"] + info["chunk_stores"]) * cb
            moved += (info["partial_loads"] + info["partial_stores"]) * (cb // workloads.ELEM_BYTES[w.dtype]) * 4
            if w.n_dst:
                moved += w.n_dst * w.object_bytes       # copy kernel: 1 read + (n_dst - 1) writes
            results[op] = {"ms": ms, "ms_median": ms_median, "wall_ms": wall_ms, "gbs": counted / (ms * 1e-3) / 1e9,
                           "gbs_median": counted / (ms_median * 1e-3) / 1e9, "bytes": counted, "moved": moved,
                           "moved_gbs": moved / (ms * 1e-3) / 1e9, "info": info, "status": state["rc"]}
            if n_sets > 1 and not w.n_dst:
                # launch-bound: what a caller written in C pays per call
                results[op]["c_loop"] = c_loop_host_time(hop, torch, w, obj_tables, [d[0] for d in dsts], order, op)
                # the same loop over more input sets than the library keeps recordings of (128): every call comes
                # with addresses it has not seen, as from a caller that gets fresh buffers for every request
                while len(obj_sets) < 160:
                    block = torch.stack(objs)
                    obj_sets.append([block[i] for i in range(w.n)])
                    obj_tables.append(hop.PtrTable(obj_sets[-1]))
                results[op]["c_loop_fresh"] = c_loop_host_time(hop, torch, w, obj_tables, [d[0] for d in dsts], order, op,
                                                               repeats=1600)
                del obj_sets[n_sets:], obj_tables[n_sets:]
        return w, objs, order, dsts, results

    # The headline workload runs first, on memory as a fresh process gets it: after the other workloads have
    # allocated and freed some tens of GiB, the same buffers allocated anew read 1.5 points slower (measured:
    # 84.4 % of the HBM peak first, 82.9 % last, whatever the number of warm-up steps).
    w, objs, order, dsts, res = run_workload(args.workload, args.steps, args.warmup)
    extra = None
    if not args.skip_all_configs:
        # The other four workloads (workload 4 also without its failure), each with the bytes counted for the
        # metric, the bytes its launches really moved, and the fraction of the HBM peak on counted bytes.
        extra = {}
        for cfg, no_fail in ((1, False), (3, False), (4, False), (4, True), (5, False)):
            if cfg == args.workload and not no_fail:
                continue
            # the tiny workloads are launch-bound: median over batches of 100 calls (see time_calls_median)
            tiny = cfg in (1, 5)
            wk, o2, _, d2, rs = run_workload(cfg, 1000 if tiny else 50, 300 if tiny else 20, no_fail,
                                             time_calls_median if tiny else time_calls)
            for opn, rr in rs.items():
                t = profiled_traffic(wk.name, hop.hop_kernel_config())
                extra["%s/%s" % (wk.name, opn)] = {
                    "GB/s": round(rr["gbs_median"], 2), "ms": round(rr["ms_median"], 5), "ms_mean": round(rr["ms"], 5),
                    "frac_of_hbm_peak": round(rr["gbs_median"] / HBM_PEAK_GBS, 4), "counted_bytes": rr["bytes"],
                    "counted_as": "(k_eff + n_dst) x object_bytes" if wk.n_dst else "(k_eff + 1) x object_bytes",
                    "moved_bytes": rr["moved"], "moved_over_counted": round(rr["moved"] / rr["bytes"], 4),
                    "GB/s_moved": round(rr["moved"] / (rr["ms_median"] * 1e-3) / 1e9, 2),
                    "traffic_from_counters": t["bytes_per_call"] if t else None,
                    "status": rr["status"], "status_text": hop.hop_strerror(rr["status"]), "k_eff": rr["info"]["k_eff"],
                    "launches": rr["info"]["n_launches"], "host_ms_per_call": round(rr["wall_ms"], 5),
                    "c_caller": rr.get("c_loop"),
                    "c_caller_fresh_buffers": rr.get("c_loop_fresh"),
                    "timing": "median of batches of 100 calls" if tiny else "median of batches of 10 calls"}
            del o2, d2
            torch.cuda.empty_cache()
    op = w.ops[0]
    r = res[op]
    traffic = profiled_traffic(w.name, hop.hop_kernel_config())
    out = {
        "metric": "reduce input GB/s and % of MI355X HBM peak, N-way chunked reduce",
        "value": round(r["gbs"], 2),
        "unit": "GB/s",
        "pct_of_hbm_peak": round(100.0 * r["gbs"] / HBM_PEAK_GBS, 2),
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(r["ms"], 5),
        "ms_per_step_median": round(r["ms_median"], 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": {"f32": "f32", "bf16": "bf16 in, f32 accumulate", "i32": "int32"}[w.dtype],
        "data": "synthetic",
        "config": {"workload": w.name, "n": w.n, "k": w.k, "object_bytes": w.object_bytes,
                   "chunk_bytes": w.chunk_bytes, "tree_degree": r["info"]["degree_used"], "op": op,
                   "counted_bytes": r["bytes"], "launches_per_step": r["info"]["n_launches"],
                   "host_ms_per_step": round(r["wall_ms"], 5)},
        # one launch per call for this workload: the kernel's average duration over the timed region is the
        # time per call (the gap between launches, under 1 % here, counts against the kernel)
        "roofline": {"bound": "hbm", "achieved": round(r["gbs"], 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(r["gbs"] / HBM_PEAK_GBS, 4),
                     "traffic": traffic["bytes_per_call"] if traffic else None,
                     "traffic_source": (traffic["profile"] if traffic else None),
                     "kernel": "hop::reduce_kernel_inline", "per_unit": "(k_eff+1) x object_bytes per launch"},
        "paper_context": PAPER_CONTEXT,
    }
    if extra is not None:
        out["all_configs"] = extra
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
        ms, _, _ = time_calls(probe, 10, 2, torch)
        out["copy_probe"] = {"bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4, "ms": round(ms, 5),
                             "GB/s_read_plus_write": round(2 * src.numel() * 4 / (ms * 1e-3) / 1e9, 2),
                             "kernel": "hop::copy_kernel"}
        del src, dstp
    if args.degree_sweep:
        sweep = {}
        table = hop.PtrTable(objs)
        for deg in sorted({1, 2, 4, 8, w.k}):
            st = {"i": 0, "info": None}

            def step_deg():
                st["i"] += 1
                _, st["info"] = hop.hop_reduce(dsts[st["i"] & 1][0], table, w.k, op, w.dtype, w.chunk_bytes, deg, order,
                                               None)
            ms, _, _ = time_calls(step_deg, max(20, args.steps // 4), 10, torch)
            nbytes = (st["info"]["k_eff"] + 1) * w.object_bytes        # reduce only, nobody fails
            sweep["d=%d" % deg] = {"ms": round(ms, 5), "GB/s": round(nbytes / (ms * 1e-3) / 1e9, 1),
                                   "levels": st["info"]["stack_depth"]}
        rc_cal, lat, bw = hop.hop_calibrate()
        sweep["calibrated"] = {"status": rc_cal, "latency_us": round(lat * 1e6, 3), "GB/s": round(bw / 1e9, 1)}
        sweep["picked_by_eq1"] = hop.hop_pick_degree(w.k, w.object_bytes, 0.0, 0.0)
        out["degree_sweep"] = sweep
    if args.size_sweep:
        import statistics
        rows = []
        for mib in (1, 2, 3, 4, 6, 8, 10, 12, 16, 24, 32, 64):
            ws = w.scaled(mib << 20, min(w.chunk_bytes, mib << 20), fail={}, name="%s_%dMiB" % (w.name, mib))
            n_sets = max(2, -(-(768 << 20) // (w.n * (mib << 20))))          # three times the memory-side cache
            base = workloads.make_objects(ws, device=dev)
            sets = [hop.PtrTable(base)]
            for _ in range(n_sets - 1):
                block = torch.stack(base)
                sets.append(hop.PtrTable([block[i] for i in range(ws.n)]))
            dd = [torch.empty_like(base[0]) for _ in range(2)]
            stt = {"i": 0}
            strm = torch.cuda.current_stream().cuda_stream

            def step_size():
                stt["i"] += 1
                hop.hop_reduce(dd[stt["i"] & 1], sets[stt["i"] % n_sets], ws.k, op, ws.dtype, ws.chunk_bytes, ws.tree_degree,
                               order, None, stream=strm)
            reps = 400 if mib <= 8 else 100
            ms, _, med = time_calls_median(step_size, reps, 50, torch, batch=max(10, reps // 10))
            nbytes = (ws.k + 1) * ws.object_bytes
            rows.append({"MiB": mib, "us": round(med * 1e3, 2), "GB/s": round(nbytes / (med * 1e-3) / 1e9, 1),
                         "frac": round(nbytes / (med * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "bytes": nbytes})
            del base, sets, dd
            torch.cuda.empty_cache()
        # least squares of time against bytes over the sizes
        xs = [r["bytes"] for r in rows]
        ys = [r["us"] for r in rows]
        mx, my = statistics.mean(xs), statistics.mean(ys)
        slope = sum((x - mx) * (y - my) for x, y in zip(xs, ys)) / sum((x - mx) ** 2 for x in xs)
        fixed = my - slope * mx
        out["size_sweep"] = {"rows": rows, "fit": {"fixed_us": round(fixed, 2), "rate_GB/s": round(1e-3 / slope, 1),
                                                  "model": "us = fixed_us + bytes / rate"}}
        for r in rows:
            r["model_us"] = round(fixed + slope * r["bytes"], 2)
    if args.many_objects_sweep:
        # many inputs of small to medium size (sum, 16-ary tree), inputs not in any cache: which of the
        # library's forms of a long program takes the call depends on inputs x size
        sweep_dt = args.many_objects_dtype
        base5 = workloads.WORKLOADS[{"f32": 5, "bf16": 4, "i32": 3}[sweep_dt]]
        tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "i32": torch.int32}[sweep_dt]
        es = workloads.ELEM_BYTES[sweep_dt]
        rows = []
        for n_in in (128, 256, 1000, 4000):
            for nbytes in (1 << 10, 4 << 10, 16 << 10, 64 << 10, 256 << 10, 1 << 20):
                if n_in * nbytes > (1 << 30):
                    continue
                ws = base5.scaled(nbytes, nbytes, n=n_in, k=n_in, tree_degree=16, fail={}, name="many_%d_%d" % (n_in, nbytes),
                                  n_dst=0)
                n_sets = max(4, min(64, (256 << 20) // (n_in * nbytes)))
                sets = []
                for _ in range(n_sets):
                    block = (torch.rand((n_in, nbytes // es), device=dev) * 64).to(tdt)
                    t = hop.PtrTable([block[i] for i in range(n_in)])
                    t.keep = block
                    sets.append(t)
                dd = [torch.zeros(nbytes // es, device=dev, dtype=tdt) for _ in range(2)]
                so = ws.ready_order()
                stt = {"i": 0, "info": None}
                strm = torch.cuda.current_stream().cuda_stream

                def step_many():
                    stt["i"] += 1
                    _, stt["info"] = hop.hop_reduce(dd[stt["i"] & 1], sets[stt["i"] % n_sets], ws.k, "sum", ws.dtype, ws.chunk_bytes,
                                                    ws.tree_degree, so, None, stream=strm)
                reps = 400 if n_in * nbytes < (64 << 20) else 60
                _, _, med = time_calls_median(step_many, reps, max(2 * n_sets, 50), torch, batch=max(10, reps // 10))
                counted = (n_in + 1) * nbytes
                rows.append({"inputs": n_in, "object_bytes": nbytes, "us": round(med * 1e3, 2),
                             "GB/s": round(counted / (med * 1e-3) / 1e9, 1), "launches": stt["info"]["n_launches"]})
                del sets, dd
                torch.cuda.empty_cache()
        out["many_objects_sweep"] = {"dtype": sweep_dt, "rows": rows}
    if args.streamed_interval_us is not None:
        out["streamed_chunks"] = streamed_chunks(hop, torch, w, objs, order, dsts[0][0], args.streamed_interval_us)
    if args.paced_interval_us is not None:
        out["paced_arrivals"] = paced_arrivals(hop, torch, w, objs, order, dsts[0][0], args.paced_interval_us)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
