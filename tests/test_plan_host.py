"""Host-side checks of the library (no GPU): it loads, exports its ABI, and its
scheduler + accumulator programs reproduce the oracle when interpreted in numpy."""
import ctypes
import math
import os
import re

import numpy as np
import pytest

import oracle
import paper_2002_05814_amd as hop
import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
NP_OP = {
    "sum": lambda a, b: a + b,
    "min": lambda a, b: np.where(b < a, b, a),
    "max": lambda a, b: np.where(b > a, b, a),
}
ORA_OP = {"sum": oracle.SUM, "min": oracle.MIN, "max": oracle.MAX}


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "hop.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(hop_[a-z_]+)\s*\(", text))
    assert declared == set(hop.EXPORTS), declared ^ set(hop.EXPORTS)
    L = hop.lib()
    for name in declared:
        assert getattr(L, name) is not None
    assert hop.hop_strerror(0) == "ok" and "align" in hop.hop_strerror(hop.HOP_ERR_ALIGN)
    assert "captured" in hop.hop_strerror(hop.HOP_ERR_CAPTURE) and hop.HOP_ERR_CAPTURE == -8


def test_workspace_bytes_counts_every_kind_of_scratch():
    W = hop.hop_workspace_bytes
    MiB = 1 << 20
    # workload 2: program in the kernel arguments, one destination: nothing from the workspace
    assert W(16, 12, 64 * MiB, 4 * MiB, 4, "f32") == 0
    # workload 3: the table of the other 63 destinations rides in the kernel arguments; 99 others are staged
    assert W(64, 64, 16 * MiB, MiB, 2, "i32", n_dst=64) == 0
    assert W(64, 64, 16 * MiB, MiB, 2, "i32", n_dst=100) == 256 << 10
    # a program of 200 steps over large objects is staged
    assert W(200, 200, 2 * MiB, MiB, 4, "f32") == 256 << 10
    # workload 5: 56 sub-programs with one 4 KiB partial result each, and their records
    w5 = W(1024, 1000, 4096, 4096, 16, "f32")
    assert 56 * 4096 < w5 <= 512 << 10
    # workload 4 with failures possible: three kept partial results of 4 bytes per element
    assert W(32, 32, 256 * MiB, 8 * MiB, 8, "bf16", policy=hop.HOP_WS_FAILURES) == 3 * 512 * MiB
    assert W(32, 32, 256 * MiB, 8 * MiB, 1, "bf16", policy=hop.HOP_WS_FAILURES) == 0           # a chain has no subtrees
    assert W(32, 32, MiB, 64 << 10, 8, "bf16", policy=hop.HOP_WS_FAILURES) == 0                 # too small to keep anything
    # eager sessions: one array of saved accumulators per level (2 for this tree) and a block of staged segments
    assert W(16, 12, 64 * MiB, 4 * MiB, 4, "f32", policy=hop.HOP_WS_EAGER) == 2 * 64 * MiB + (256 << 10)
    assert W(64, 64, 32 * MiB, MiB, 2, "bf16", policy=hop.HOP_WS_EAGER) == 5 * 64 * MiB + (256 << 10)
    # invalid shapes
    assert W(4, 5, 64, 16, 2, "f32") == 0 and W(4, 2, 64, 24, 2, "f32") == 0


def test_info_struct_layout_matches_header():
    # int32 x4, int64, int32 x2, int64 x4 -> 64 bytes with natural alignment
    assert ctypes.sizeof(hop.HopInfo) == 64
    assert hop.HopInfo.chunks_redone.offset == 16 and hop.HopInfo.partial_stores.offset == 56
    assert ctypes.sizeof(hop.PlanEntry) == 12 and ctypes.sizeof(hop.PlanLaunch) == 48


@pytest.mark.parametrize("d", [1, 2, 3, 4, 8, 16, 1 << 20])
def test_slots_match_oracle(d):
    for k in list(range(1, 70)) + [1000, 4097]:
        rc, got = hop.hop_plan_slots(k, d)
        want, _ = oracle.tree_slots(k, d)
        assert rc == hop.HOP_OK and np.array_equal(got, want), (k, d)


def interpret(objs, launches, entries, n_elems, chunk_elems, op):
    """Apply the recorded launches in order, exactly as the header describes them: steps
    [step_begin, step_end) of the program in force, accumulators restored from / saved to a
    per-level spill array between segments, the result stored by final launches."""
    f = NP_OP[op]
    dst = np.zeros(n_elems, objs[0].dtype)
    spill = {}
    kept = {}                # q -> array of kept partial results; NaN / a marker where nothing was kept
    for c0, c1, e0, e1, t0, t1, final, live_before, live_after in launches:
        seg = slice(c0 * chunk_elems, min(c1 * chunk_elems, n_elems))
        prog = entries[e0:e1]
        assert 0 <= t0 <= t1 <= len(prog) and (final == (t1 == len(prog))) and (t0 < t1 or final)
        assert (live_before == 0) == (t0 == 0)
        acc = {L: spill[L][seg].copy() for L in range(live_before)}
        stored_now = {}
        for e in prog[t0:t1]:
            obj, level, is_set, n_fold = e[:4]
            if obj >= 0:
                x = objs[obj][seg]
            else:
                # a kept partial result: it must have been stored for every one of these chunks by an
                # earlier launch (never by this one)
                assert t0 == 0 and final
                have, x = kept[-obj - 1]
                assert have[c0:c1].all(), "reads a partial that was never kept"
                x = x[seg]
            acc[level] = x.copy() if is_set else f(acc[level], x).astype(x.dtype)
            if len(e) > 4:
                q, save_level = e[4], e[5]
                assert t0 == 0 and final and save_level <= level and level - save_level <= n_fold
                while level > save_level:
                    acc[level - 1] = f(acc[level - 1], acc[level]).astype(x.dtype)
                    del acc[level]
                    level -= 1
                    n_fold -= 1
                stored_now[q] = acc[level].copy()
            for _ in range(n_fold):
                acc[level - 1] = f(acc[level - 1], acc[level]).astype(x.dtype)
                del acc[level]
                level -= 1
        for q, val in stored_now.items():
            have, arr = kept.setdefault(q, (np.zeros(max(c1, 1) + 10 ** 6, bool), np.zeros(n_elems, objs[0].dtype)))
            have[c0:c1] = True
            arr[seg] = val
        if final:
            assert list(acc) == [0] and live_after == 0
            dst[seg] = acc[0]
        else:
            assert sorted(acc) == list(range(live_after))
            for L in range(live_after):
                spill.setdefault(L, np.zeros(n_elems, objs[0].dtype))[seg] = acc[L]
    return dst


def random_case(rng, max_n=14, with_fail=True):
    n = int(rng.integers(1, max_n + 1))
    k = int(rng.integers(1, n + 1))
    d = int(rng.choice([1, 2, 3, 4, 8, n + 5]))
    chunk_elems = 4 * int(rng.integers(1, 5))
    n_elems = int(rng.integers(1, 6 * chunk_elems))
    C = -(-n_elems // chunk_elems)
    order = rng.permutation(n).astype(np.int32)
    fm = None
    if with_fail and rng.random() < 0.7:
        fm = np.full(n, -1, np.int64)
        bad = rng.random(n) < 0.35
        fm[bad] = rng.integers(0, C + 2, size=int(bad.sum()))
    return n, k, d, chunk_elems, n_elems, order, fm


# The schedule is in units of chunks, so the same plan can be made for objects 2^20 times as large
# (chunks of megabytes instead of bytes) and still be interpreted on the small arrays: that is how the
# tests here reach the policies that depend on the size of a launch (partial results are kept only by
# launches over at least 8 MiB per object).
BIG = 1 << 20


@pytest.mark.parametrize("op", ["sum", "max", "min"])
@pytest.mark.parametrize("scale", [1, BIG])
def test_interpreted_plan_equals_oracle_f32(op, scale):
    rng = np.random.default_rng({"sum": 1, "max": 2, "min": 3}[op] + (scale > 1) * 10)
    n_kept = n_reused = 0
    for _ in range(300):
        n, k, d, ce, E, order, fm = random_case(rng, max_n=14 if scale == 1 else 30)
        objs = [(rng.standard_normal(E) * 10.0 ** rng.integers(-3, 4)).astype(np.float32) for _ in range(n)]
        rc, info, launches, entries = hop.hop_plan_reduce(n, E * 4 * scale, k, "f32", ce * 4 * scale, d, order, fm)
        n_kept += info["partial_stores"] > 0
        n_reused += info["partial_loads"] > 0
        orc, want, k_eff, n_rep = oracle.reduce(objs, k, ORA_OP[op], oracle.F32, ce, d, order, fm)
        assert rc == orc, (rc, orc)
        if rc < 0:
            assert rc == hop.HOP_ERR_NO_SURVIVOR
            continue
        assert info["k_eff"] == k_eff and info["n_replaced"] == n_rep and info["degree_used"] == d
        got = interpret(objs, launches, entries, E, ce, op)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
        # every object in the final program exactly once; k_eff of them
        final = entries[launches[-1][2]:launches[-1][3]]
        assert launches[-1][6] == 1 and max(e[1] for e in final) + 1 <= info["stack_depth"] <= hop.HOP_MAX_DEPTH
        if not any(e[0] < 0 for e in final):
            assert len(final) == k_eff and len({e[0] for e in final}) == k_eff
    # small launches never keep anything; large ones with mid-stream failures do, and reuse it
    assert (n_kept, n_reused) == (0, 0) if scale == 1 else (n_kept > 20 and n_reused > 10), (n_kept, n_reused)


def test_interpreted_plan_equals_oracle_i32_wrapping():
    rng = np.random.default_rng(4)
    for _ in range(100):
        n, k, d, ce, E, order, fm = random_case(rng)
        objs = [rng.integers(-2 ** 31, 2 ** 31, size=E, dtype=np.int64).astype(np.int32) for _ in range(n)]
        scale = BIG if _ % 2 else 1
        rc, info, launches, entries = hop.hop_plan_reduce(n, E * 4 * scale, k, "i32", ce * 4 * scale, d, order, fm)
        orc, want, _, _ = oracle.reduce(objs, k, oracle.SUM, oracle.I32, ce, d, order, fm)
        assert rc == orc
        if rc < 0:
            continue
        with np.errstate(over="ignore"):
            got = interpret([o.view(np.uint32) for o in objs], launches, entries, E, ce, "sum")
        assert np.array_equal(got.view(np.int32), want)


def run_entries(objs, entries, op, partials=()):
    f = NP_OP[op]
    acc = {}
    for obj, level, is_set, n_fold in entries:
        x = objs[obj] if obj >= 0 else partials[-obj - 1]
        acc[level] = x.copy() if is_set else f(acc[level], x).astype(x.dtype)
        for _ in range(n_fold):
            acc[level - 1] = f(acc[level - 1], acc[level]).astype(x.dtype)
            del acc[level]
            level -= 1
    assert list(acc) == [0]
    return acc[0]


def run_plan_passes(objs, tops, subs, op):
    """Evaluate sub-programs pass by pass (each reads only partials of earlier passes), then the top."""
    partials = [None] * len(subs)
    for p in range(1 + max([ps for ps, _ in subs], default=-1)):
        for g, (ps, steps) in enumerate(subs):
            if ps == p:
                for e in steps:
                    assert e[0] >= 0 or (subs[-e[0] - 1][0] < p and partials[-e[0] - 1] is not None)
                partials[g] = run_entries(objs, steps, op, partials)
    return run_entries(objs, tops, op, partials)


@pytest.mark.parametrize("want_steps,min_run,max_run", [(1, 1, 1000), (1, 2, 5), (8, 4, 16), (64, 4, 64), (30, 9, 20), (2, 1, 3)])
def test_split_program_keeps_the_bits(want_steps, min_run, max_run):
    rng = np.random.default_rng(want_steps * 10 + min_run)
    n_split = 0
    for _ in range(120):
        n = int(rng.integers(1, 200))
        k = int(rng.integers(1, n + 1))
        d = int(rng.choice([1, 2, 3, 4, 16, n + 1]))
        E = 16
        order = rng.permutation(n).astype(np.int32)
        fm = None
        if rng.random() < 0.5:
            fm = np.full(n, -1, np.int64)
            bad = rng.random(n) < 0.2
            fm[bad] = rng.integers(0, 3, size=int(bad.sum()))
        objs = [(rng.standard_normal(E) * 10.0 ** rng.integers(-3, 4)).astype(np.float32) for _ in range(n)]
        rc, info, launches, entries = hop.hop_plan_reduce(n, E * 4, k, "f32", 32, d, order, fm)
        if rc < 0:
            continue
        final = entries[launches[-1][2]:launches[-1][3]]
        src, tops, subs = hop.hop_plan_split(final, want_steps, min_run, max_run)
        whole = run_entries(objs, final, "sum")
        if src == hop.HOP_PARTIAL:
            assert subs == [] and tops == final
            continue
        n_split += 1
        # every object still exactly once; every partial used exactly once
        seen = [e[0] for e in tops if e[0] >= 0] + [e[0] for _, sp in subs for e in sp if e[0] >= 0]
        assert sorted(seen) == sorted(e[0] for e in final)
        refs = [-e[0] - 1 for e in tops if e[0] < 0] + [-e[0] - 1 for _, sp in subs for e in sp if e[0] < 0]
        assert sorted(refs) == list(range(len(subs)))
        got = run_plan_passes(objs, tops, subs, "sum")
        assert np.array_equal(got.view(np.uint32), whole.view(np.uint32))
        # sub-programs respect the length limits
        assert all(min_run <= len(sp) <= max_run for _, sp in subs)
    assert n_split > 10
    # workload 5: 1000 steps in one program become one pass of short programs and a short top program
    w = workloads.WORKLOADS[5]
    _, _, launches, entries = hop.hop_plan_reduce(w.n, w.object_bytes, w.k, w.dtype, w.chunk_bytes, w.tree_degree,
                                                  w.ready_order(), None)
    src, tops, subs = hop.hop_plan_split(entries, 128, 4, 64)
    assert src == hop.HOP_OK and len(tops) < 128 and max(len(sp) for _, sp in subs) <= 64
    assert {ps for ps, _ in subs} == {0}
    assert len(tops) + sum(len(sp) for _, sp in subs) - len(subs) == 1000
    # a binary tree on 4000 inputs needs a second round of cutting
    _, _, _, e2 = hop.hop_plan_reduce(4000, 64, 4000, "f32", 64, 2, None, None)
    src, tops, subs = hop.hop_plan_split(e2, 128, 4, 64)
    assert src == hop.HOP_OK and len(tops) < 128 and {ps for ps, _ in subs} == {0, 1}
    assert len(tops) + sum(len(sp) for _, sp in subs) - len(subs) == 4000


def run_chains(objs, chains, op):
    """Chains pass by pass: each reads only objects and values of chains of earlier passes; the last one is the result."""
    f = NP_OP[op]
    values = [None] * len(chains)
    for p in range(1 + max(ps for ps, _ in chains)):
        for g, (ps, items) in enumerate(chains):
            if ps != p:
                continue
            vals = []
            for it in items:
                if it < 0:
                    assert chains[-it - 1][0] < p and values[-it - 1] is not None
                vals.append(objs[it] if it >= 0 else values[-it - 1])
            acc = vals[0].copy()
            for x in vals[1:]:
                acc = f(acc, x).astype(x.dtype)
            values[g] = acc
    return values[-1]


@pytest.mark.parametrize("min_cut", [1, 2, 4, 9])
def test_program_as_chains_keeps_the_bits(min_cut):
    rng = np.random.default_rng(40 + min_cut)
    n_cut = 0
    for _ in range(150):
        n = int(rng.integers(1, 200))
        k = int(rng.integers(1, n + 1))
        d = int(rng.choice([1, 2, 3, 4, 16, n + 1]))
        order = rng.permutation(n).astype(np.int32)
        fm = None
        if rng.random() < 0.5:
            fm = np.full(n, -1, np.int64)
            bad = rng.random(n) < 0.2
            fm[bad] = rng.integers(0, 3, size=int(bad.sum()))
        objs = [(rng.standard_normal(16) * 10.0 ** rng.integers(-3, 4)).astype(np.float32) for _ in range(n)]
        rc, info, launches, entries = hop.hop_plan_reduce(n, 64, k, "f32", 32, d, order, fm)
        if rc < 0:
            continue
        final = entries[launches[-1][2]:launches[-1][3]]
        max_items = int(rng.choice([2, 3, 8, 23, 1000]))
        src, chains = hop.hop_plan_chains(final, min_cut, max_items)
        if len(final) < 2:
            assert src == hop.HOP_PARTIAL and chains == []
            continue
        assert src == hop.HOP_OK
        # every object exactly once, every chain's value used exactly once except the last one's
        seen = [it for _, items in chains for it in items if it >= 0]
        assert sorted(seen) == sorted(e[0] for e in final)
        refs = [-it - 1 for _, items in chains for it in items if it < 0]
        assert sorted(refs) == list(range(len(chains) - 1))
        # a chain's pass is one more than the latest pass it reads from, 0 if it reads objects only
        for ps, items in chains:
            assert ps == max([0] + [chains[-it - 1][0] + 1 for it in items if it < 0]) and 2 <= len(items) <= max_items
        whole = run_entries(objs, final, "sum")
        got = run_chains(objs, chains, "sum")
        assert np.array_equal(got.view(np.uint32), whole.view(np.uint32))
        n_cut += len(chains) > 1
    assert n_cut > 30
    # workload 5: 1000 steps become three passes whose longest chains have 18, 17 and 16 items, with at
    # most 59 chains in a pass (a workgroup evaluates 64 side by side)
    w = workloads.WORKLOADS[5]
    _, _, launches, entries = hop.hop_plan_reduce(w.n, w.object_bytes, w.k, w.dtype, w.chunk_bytes, w.tree_degree,
                                                  w.ready_order(), None)
    src, chains = hop.hop_plan_chains(entries, 4)
    assert src == hop.HOP_OK
    per_pass = {}
    for ps, items in chains:
        per_pass.setdefault(ps, []).append(len(items))
    assert sorted(per_pass) == [0, 1, 2] and [max(per_pass[p]) for p in range(3)] == [18, 17, 16]
    assert [len(per_pass[p]) for p in range(3)] == [59, 3, 1]
    # a chain or a star is one fold with nothing to do side by side: a single chain, or, with a limit on
    # the items of a chain, pieces that follow each other one pass each
    for d in (1, 5000):
        _, _, _, e1 = hop.hop_plan_reduce(300, 64, 300, "f32", 64, d, None, None)
        src, chains = hop.hop_plan_chains(e1, 4, 1000)
        assert src == hop.HOP_OK and len(chains) == 1 and len(chains[0][1]) == 300
        src, chains = hop.hop_plan_chains(e1, 4, 23)
        assert src == hop.HOP_OK and [p for p, _ in chains] == list(range(14))
        assert [len(items) for _, items in chains] == [23] * 13 + [1 + 300 - 23 - 12 * 22]
    # programs that read kept partial results have no such form
    assert hop.hop_plan_chains([(0, 0, 1, 0), (-1, 0, 0, 0)], 4)[0] == hop.HOP_PARTIAL
    assert hop.hop_plan_chains([(0, 0, 1, 0, 0, 0), (1, 0, 0, 0)], 4)[0] == hop.HOP_PARTIAL


def test_failure_free_call_is_one_launch_over_all_chunks():
    for cfg in (1, 2, 3, 5):
        w = workloads.WORKLOADS[cfg]
        rc, info, launches, entries = hop.hop_plan_reduce(w.n, w.object_bytes, w.k, w.dtype, w.chunk_bytes,
                                                          w.tree_degree, w.ready_order(), w.fail_mask())
        assert rc == hop.HOP_OK and info["k_eff"] == w.k and info["chunks_redone"] == 0
        assert launches == [(0, w.n_chunks, 0, w.k, 0, w.k, 1, 0, 0)] and info["n_launches"] == 1
        # only the first k arrivals are ever read
        assert sorted(e[0] for e in entries) == sorted(w.ready_order()[:w.k].tolist())
    # accumulator levels needed: 2, 2, 3 for workloads 1, 2, 5; workload 3 picks a degree from {1, 2, k}
    depths = {}
    for cfg in (1, 2, 3, 5):
        w = workloads.WORKLOADS[cfg]
        _, info, _, _ = hop.hop_plan_reduce(w.n, w.object_bytes, w.k, w.dtype, w.chunk_bytes, w.tree_degree,
                                            w.ready_order(), None)
        depths[cfg] = (info["stack_depth"], info["degree_used"])
    assert depths[1] == (2, 2) and depths[2] == (2, 4) and depths[5] == (3, 16)
    assert depths[3][1] in (1, 2, 64)


def test_mid_stream_failure_repairs_from_kept_subtree_partials():
    w = workloads.WORKLOADS[4]          # participant 7 fails after its 10th chunk of 32
    rc, info, launches, entries = hop.hop_plan_reduce(w.n, w.object_bytes, w.k, w.dtype, w.chunk_bytes,
                                                      w.tree_degree, w.ready_order(), w.fail_mask())
    assert rc == hop.HOP_PARTIAL and info["k_eff"] == 31 and info["n_failed_seen"] == 1
    assert info["n_replaced"] == 0 and info["stack_depth"] == 2
    # chunks 0..9 are produced with all 32 participants while any of them can still fail: the launch
    # also keeps the partial results of the three subtrees below the root (9, 9 and 8 arrivals). #7 is
    # the 29th arrival, a childless child of the root: the repair of chunks 0..9 reads the three kept
    # partials, the root's own object and its four remaining childless children; chunks 10..31 are
    # produced from the 31 survivors.
    assert [(l[0], l[1]) for l in launches] == [(0, 10), (0, 10), (10, 32)]
    first, repair, rest = (entries[l[2]:l[3]] for l in launches)
    assert len(first) == 32 and 7 in {e[0] for e in first}
    assert [e[4] for e in first if len(e) > 4] == [0, 1, 2] and [first.index(e) for e in first if len(e) > 4] == [8, 18, 26]
    assert [e[0] for e in repair if e[0] < 0] == [-1, -2, -3] and len(repair) == 3 + 1 + 4
    assert 7 not in {e[0] for e in repair} and all(len(e) == 4 for e in repair + rest)
    assert len(rest) == 31 and 7 not in {e[0] for e in rest}
    assert info["n_launches"] == 3 and info["chunks_redone"] == 10 * 5
    assert info["chunk_steps"] == 10 * 32 + 10 * 5 + 22 * 31 and info["chunk_stores"] == 10 + 10 + 22
    assert info["partial_stores"] == 10 * 3 and info["partial_loads"] == 10 * 3
    # the survivors keep their relative order
    assert [e[0] for e in rest] == [e[0] for e in first if e[0] != 7]
    # the failure time changes the repair work, never the final program
    for c in (1, 5, 31):
        fm = w.fail_mask().copy()
        fm[7] = c
        _, info_c, launches_c, entries_c = hop.hop_plan_reduce(w.n, w.object_bytes, w.k, w.dtype, w.chunk_bytes,
                                                               w.tree_degree, w.ready_order(), fm)
        assert [(l[0], l[1]) for l in launches_c] == [(0, c), (0, c), (c, 32)]
        assert entries_c[launches_c[2][2]:launches_c[2][3]] == rest
        assert info_c["chunks_redone"] == c * 5
    # a participant inside a subtree: that subtree is read again, the other two come from their partials
    order = w.ready_order()
    inside = int(order[12])                  # 13th arrival: in the second subtree (arrivals 11..19)
    fm = np.full(w.n, -1, np.int64)
    fm[inside] = 4
    _, info_i, launches_i, entries_i = hop.hop_plan_reduce(w.n, w.object_bytes, w.k, w.dtype, w.chunk_bytes,
                                                           w.tree_degree, order, fm)
    repair_i = entries_i[launches_i[1][2]:launches_i[1][3]]
    assert [e[0] for e in repair_i if e[0] < 0] == [-1, -3] and len(repair_i) == 2 + 1 + 8 + 5
    assert info_i["chunks_redone"] == 4 * 14
    # small launches (at most 1 MiB per object) keep nothing: the chunks are produced again whole
    ws = w.scaled((1 << 20) + 6, 32 << 10)
    _, info_s, launches_s, _ = hop.hop_plan_reduce(ws.n, ws.object_bytes, ws.k, ws.dtype, ws.chunk_bytes,
                                                   ws.tree_degree, ws.ready_order(), ws.fail_mask())
    assert [(l[0], l[1]) for l in launches_s] == [(0, 10), (0, 33)] and info_s["partial_stores"] == 0
    assert info_s["chunks_redone"] == 10 * 31


def test_deep_tree_keeps_partials_of_a_lower_level():
    # binary tree over 32 fp32 objects of 64 MiB in 8 MiB chunks: the two subtrees below the root hold 16
    # and 15 arrivals, so a repair from them would read half of the objects again. The four subtrees two
    # levels down make the expected repair smaller.
    n = k = 32
    fm = np.full(n, -1, np.int64)
    fm[19] = 3                               # the 20th arrival fails after 3 chunks
    rc, info, launches, entries = hop.hop_plan_reduce(n, 64 << 20, k, "f32", 8 << 20, 2, None, fm)
    assert rc == hop.HOP_PARTIAL and info["k_eff"] == 31 and info["stack_depth"] == 4
    assert [(l[0], l[1]) for l in launches] == [(0, 3), (0, 3), (3, 8)]
    first, repair, rest = (entries[l[2]:l[3]] for l in launches)
    saves = [(first.index(e), e[4], e[5]) for e in first if len(e) > 4]
    # four kept values, each stored from the accumulator level its subtree's result sits at
    assert [s[1] for s in saves] == [0, 1, 2, 3] and len({s[0] for s in saves}) == 4
    assert saves[-1][0] == 31 - 0 and saves[0][0] == 7          # in-order: the last subtree ends the program
    # the repair reads three kept values and the surviving objects of the fourth subtree and outside
    kept_read = [e[0] for e in repair if e[0] < 0]
    assert len(kept_read) == 3 and 19 not in {e[0] for e in repair}
    assert len(repair) < 16 and info["chunks_redone"] == 3 * (len(repair) - 3)
    assert info["partial_stores"] == 3 * 4 and info["partial_loads"] == 3 * 3
    # numerically: the launches applied in order (the repair reading what the first one kept) give the
    # oracle's result over the 31 survivors, bit for bit; 4 elements stand for each 8 MiB chunk
    rng = np.random.default_rng(5)
    objs = [(rng.standard_normal(32) * 10.0 ** rng.integers(-3, 4)).astype(np.float32) for _ in range(n)]
    got = interpret(objs, launches, entries, 32, 4, "sum")
    orc, want, _, _ = oracle.reduce(objs, k, oracle.SUM, oracle.F32, 4, 2, None, fm)
    assert orc == rc and np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_replacement_from_waiting_objects():
    # 6 of 10, second arrival fails after 3 chunks of 8: the 7th arrival takes its place
    n, k, C = 10, 6, 8
    fm = np.full(n, -1, np.int64)
    fm[1] = 3
    rc, info, launches, entries = hop.hop_plan_reduce(n, C * 64, k, "f32", 64, 2, None, fm)
    assert rc == hop.HOP_OK and info["n_replaced"] == 1 and info["k_eff"] == 6
    final = entries[launches[-1][2]:launches[-1][3]]
    assert [e[0] for e in final] == [0, 6, 2, 3, 4, 5]
    assert [(l[0], l[1]) for l in launches] == [(0, 3), (0, 8)]


def test_pick_degree_is_argmin_of_eq1_over_1_2_n():
    def T(n, d, S, L, B):
        return n * L + S / B if d == 1 else L * math.log(n) / math.log(d) + d * S / B
    rng = np.random.default_rng(8)
    for _ in range(300):
        n = int(rng.integers(3, 200))
        S = int(10 ** rng.uniform(2, 10))
        L = 10 ** rng.uniform(-7, -2)
        B = 10 ** rng.uniform(8, 13)
        got = hop.hop_pick_degree(n, S, L, B)
        costs = {d: T(n, d, S, L, B) for d in (1, 2, n)}
        best = min(costs.values())
        assert got in costs and costs[got] <= best * 1.02
        # within 2 % of the best the tree with the fewest accumulator levels wins (chain and star: one level)
        if got == 2:
            assert min(costs[1], costs[n]) > best * 1.02
        elif costs[got] > best * (1 + 1e-12):
            assert costs[2] == best
    # the qualitative rule of the paper's appendix B on its own testbed (10 Gbps, ~0.2 ms hops):
    # small objects -> d = n, large objects -> d = 1
    assert hop.hop_pick_degree(16, 1 << 10, 2e-4, 1.25e9) == 16
    assert hop.hop_pick_degree(16, 1 << 30, 2e-4, 1.25e9) == 1
    # a near-tie between the binary tree and the chain goes to the chain (one accumulator level):
    # T(1) = 8 L + S/B and T(2) = 3 L + 2 S/B are equal for S/B = 5 L
    assert hop.hop_pick_degree(8, 5000, 1e-6, 1e9 * 1.001) == 1
    assert hop.hop_pick_degree(8, 5000, 1e-6, 1e9 * 1.1) == 2


def test_argument_errors_without_a_device():
    P = hop.hop_plan_reduce
    assert P(0, 64, 1, "f32", 16, 2)[0] == hop.HOP_ERR_INVALID
    assert P(4, 64, 5, "f32", 16, 2)[0] == hop.HOP_ERR_INVALID
    assert P(4, 64, 0, "f32", 16, 2)[0] == hop.HOP_ERR_INVALID
    assert P(4, 64, 2, "f32", 0, 2)[0] == hop.HOP_ERR_INVALID
    assert P(4, 64, 2, "f32", 24, 2)[0] == hop.HOP_ERR_INVALID          # chunk not a multiple of 16
    assert P(4, 66, 2, "f32", 16, 2)[0] == hop.HOP_ERR_INVALID          # not a whole number of elements
    assert P(4, 66, 2, "bf16", 16, 2)[0] == hop.HOP_OK
    assert P(4, 64, 2, "f32", 16, -1)[0] == hop.HOP_ERR_INVALID
    assert P(4, 64, 2, 7, 16, 2)[0] == hop.HOP_ERR_INVALID
    assert P(4, 64, 2, "f32", 16, 2, ready_order=[0, 1, 1, 2])[0] == hop.HOP_ERR_INVALID
    assert P(4, 64, 2, "f32", 16, 2, fail_mask=[0, 0, 0, 0])[0] == hop.HOP_ERR_NO_SURVIVOR
    # a binary tree too deep for the register file of accumulators
    rc, info, _, _ = P(1 << 17, 64, 1 << 17, "f32", 16, 2)
    assert rc == hop.HOP_OK and info["stack_depth"] == hop.HOP_MAX_DEPTH
    rc, info, _, _ = P(1 << 18, 64, 1 << 18, "f32", 16, 2)
    assert rc == hop.HOP_ERR_DEPTH
    rc, info, _, _ = P(1 << 17, 64, 1 << 17, "f32", 16, 1)
    assert rc == hop.HOP_OK and info["stack_depth"] == 1


# ------------------------------------------------------------------ event-level sessions, eager segments

class SlotModel:
    """The placement rules of the header, written out independently: the t-th arrival takes position t
    (or the lowest position emptied by a failure), later arrivals wait; a failed holder is replaced
    by the first waiting object that is still alive, else its position stays empty."""

    def __init__(self, n, k, C):
        self.n, self.k, self.C = n, k, C
        self.ready = {}
        self.failed = set()
        self.slots = []              # object or None (emptied)
        self.pool = []

    def on_ready(self, obj, c):
        if obj not in self.ready:
            empties = [t for t, o in enumerate(self.slots) if o is None]
            if empties:
                self.slots[empties[0]] = obj
            elif len(self.slots) < self.k:
                self.slots.append(obj)
            else:
                self.pool.append(obj)
        self.ready[obj] = c

    def on_fail(self, obj):
        if obj in self.failed or self.ready.get(obj, 0) == self.C:
            return
        self.failed.add(obj)
        if obj in self.slots:
            t = self.slots.index(obj)
            self.pool = [p for p in self.pool if p not in self.failed]
            self.slots[t] = self.pool.pop(0) if self.pool else None

    def finish(self):
        for p in list(self.pool):
            if self.ready[p] < self.C:
                self.failed.add(p)
        for t in range(len(self.slots)):
            o = self.slots[t]
            if o is not None and self.ready[o] < self.C:
                self.on_fail(o)
        return self.slots + [None] * (self.k - len(self.slots))


def oracle_for_occupants(objs, slots, k, C, chunk_elems, d, op):
    """The oracle's value for a given final placement (None = empty position)."""
    n = len(objs)
    used = [o for o in slots if o is not None]
    spare = [i for i in range(n) if i not in used]
    order, fm = [], np.zeros(n, np.int64)
    for o in slots:
        if o is None:
            o = spare.pop()
            fm[o] = 1            # arrives, then fails with nobody alive to replace it
        else:
            fm[o] = -1
        order.append(o)
    order += spare               # fail_mask 0: they never become ready
    return oracle.reduce(objs, k, ORA_OP[op], oracle.F32, chunk_elems, d, np.array(order, np.int32), fm)


@pytest.mark.parametrize("eager,scale", [(0, 1), (1, 1), (2, 1), (5, 1), (0, BIG), (2, BIG)])
def test_random_sessions_with_segments_equal_oracle(eager, scale):
    rng = np.random.default_rng(900 + eager + (scale > 1))
    n_segmented = n_kept = n_reused = 0
    for it in range(150):
        n = int(rng.integers(2, 12 if scale == 1 else 30))
        k = int(rng.integers(1, n + 1))
        d = int(rng.choice([1, 2, 3, 4, n]))
        C = int(rng.integers(2, 7))
        ce = 4
        E = (C - 1) * ce + int(rng.integers(1, ce + 1))
        objs = [(rng.standard_normal(E) * 10.0 ** rng.integers(-2, 3)).astype(np.float32) for _ in range(n)]
        rc, s = hop.hop_plan_session_begin(n, E * 4 * scale, k, "f32", ce * 4 * scale, d)
        assert rc == hop.HOP_OK
        assert hop.hop_session_set_eager(s, eager) == hop.HOP_OK
        keeping = it % 5 != 0
        assert hop.hop_session_set_retention(s, keeping) == hop.HOP_OK
        model = SlotModel(n, k, C)
        # a random interleaving: objects arrive in random order and deliver chunks in random bursts;
        # some fail mid-stream, some never finish
        progress = {}
        arrivals = list(rng.permutation(n))
        n_never = int(rng.integers(0, 2))
        never = set(arrivals[len(arrivals) - n_never:]) if n_never else set()
        arrivals = [a for a in arrivals if a not in never]
        doomed = {int(a): int(rng.integers(0, C)) for a in arrivals if rng.random() < 0.25}
        stalls = {int(a) for a in arrivals if a not in doomed and rng.random() < 0.1}
        active = []
        while arrivals or active:
            if arrivals and (not active or rng.random() < 0.4):
                a = int(arrivals.pop(0))
                active.append(a)
                progress[a] = 0
                assert hop.hop_session_ready(s, a, 0) == hop.HOP_OK
                model.on_ready(a, 0)
                continue
            a = active[int(rng.integers(len(active)))]
            if a in doomed and progress[a] >= doomed[a]:
                assert hop.hop_session_fail(s, a) == hop.HOP_OK
                model.on_fail(a)
                active.remove(a)
                continue
            if a in stalls and progress[a] >= C - 1:
                active.remove(a)              # never delivers its last chunk
                continue
            progress[a] = min(C, progress[a] + int(rng.integers(1, 3)))
            assert hop.hop_session_ready(s, a, progress[a]) == hop.HOP_OK
            model.on_ready(a, progress[a])
            if progress[a] == C:
                active.remove(a)
        rc, info, launches, entries = hop.hop_plan_session_finish(s)
        slots = model.finish()
        live = [o for o in slots if o is not None]
        if not live:
            assert rc == hop.HOP_ERR_NO_SURVIVOR
            continue
        assert rc == (hop.HOP_OK if len(live) == k else hop.HOP_PARTIAL) and info["k_eff"] == len(live)
        final_prog = entries[launches[-1][2]:launches[-1][3]]
        if not any(e[0] < 0 for e in final_prog):
            assert [e[0] for e in final_prog] == live
        assert keeping or info["partial_stores"] == 0
        n_kept += info["partial_stores"] > 0
        n_reused += info["partial_loads"] > 0
        got = interpret(objs, launches, entries, E, ce, "sum")
        orc, want, k_eff, _ = oracle_for_occupants(objs, slots, k, C, ce, d, "sum")
        assert orc == rc and k_eff == len(live)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
        if eager == 0:
            assert all(l[4] == 0 and l[6] == 1 for l in launches)       # whole programs only
        n_segmented += any(l[6] == 0 for l in launches)
    assert n_segmented > {0: -1, 1: 30, 2: 30, 5: 0}[eager] and (eager or n_segmented == 0)
    assert (n_kept, n_reused) == (0, 0) if scale == 1 else (n_kept > 10 and n_reused > 3), (n_kept, n_reused)


def test_eager_session_overlaps_the_wait_for_the_last_arrival():
    # 8 objects of 4 chunks arrive whole, one after the other. Fused: nothing can run until the last
    # one is there, then one launch runs all 8 steps. Eager: every arrival is folded in at once, so
    # after the last arrival a single step is left.
    n, C = 8, 4
    for eager, want_last in ((0, (0, 8)), (1, (7, 8))):
        rc, s = hop.hop_plan_session_begin(n, C * 64, n, "f32", 64, 2)
        hop.hop_session_set_eager(s, eager)
        for i in range(n):
            assert hop.hop_session_ready(s, i, C) == hop.HOP_OK
            assert hop.hop_session_chunks_final(s) == (C if i == n - 1 else 0)
        rc, info, launches, entries = hop.hop_plan_session_finish(s)
        assert rc == hop.HOP_OK
        assert (launches[-1][4], launches[-1][5]) == want_last and launches[-1][6] == 1
        assert info["n_launches"] == (1 if eager == 0 else n)
        assert info["chunks_redone"] == 0


def test_failure_keeps_partials_that_never_absorbed_the_failed_object():
    # chain of 6, eager. Objects 0..3 deliver everything, object 4 delivers 2 of 4 chunks and fails,
    # object 5 is healthy. Chunks 2,3 never ran past step 4 and keep their accumulators (steps 0..3);
    # chunks 0,1 had absorbed object 4 and start over.
    n, C = 6, 4
    rc, s = hop.hop_plan_session_begin(n, C * 64, n, "f32", 64, 1)
    hop.hop_session_set_eager(s, 1)
    for i in range(4):
        hop.hop_session_ready(s, i, C)
    hop.hop_session_ready(s, 4, 2)
    hop.hop_session_ready(s, 5, C)
    assert hop.hop_session_fail(s, 4) == hop.HOP_OK
    rc, info, launches, entries = hop.hop_plan_session_finish(s)
    assert rc == hop.HOP_PARTIAL and info["k_eff"] == 5
    after = [l for l in launches if entries[l[2]:l[3]] == [(0, 0, 1, 0), (1, 0, 0, 0), (2, 0, 0, 0), (3, 0, 0, 0), (5, 0, 0, 0)]]
    # restarted chunks run all five steps, the others only the one that was missing
    assert sorted((l[0], l[1], l[4], l[5]) for l in after) == [(0, 2, 0, 5), (2, 4, 4, 5)]
    assert info["chunks_redone"] == 2 * 5


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    # there is no CPU fallback: without the built library every entry point raises
    monkeypatch.setattr(hop, "_lib", None)
    monkeypatch.setattr(hop, "LIB_PATH", str(tmp_path / "libhop.so"))
    with pytest.raises(RuntimeError, match="libhop.so is missing"):
        hop.hop_plan_slots(4, 2)
    with pytest.raises(RuntimeError):
        hop.hop_reduce(0, [], 1, "sum", "f32", 16, 2, object_bytes=0)


def test_events_before_anything_can_run_are_cheap_and_launch_nothing():
    # 3000 whole objects arrive one by one (default policy): nothing can be launched before the last
    # position is taken, one launch covers everything at the end, and the 3000 events together cost
    # far less than 3000 recompilations of a 3000-step program would (a generous wall-clock bound)
    import time
    n = 3000
    rc, s = hop.hop_plan_session_begin(n, 64, n, "f32", 64, 2)
    assert rc == hop.HOP_OK
    t0 = time.perf_counter()
    for i in range(n):
        assert hop.hop_session_ready(s, i, 1) == hop.HOP_OK
        if i in (0, 1, n // 2, n - 2):
            assert hop.hop_session_chunks_final(s) == 0
    dt = time.perf_counter() - t0
    assert hop.hop_session_chunks_final(s) == 1
    # objects beyond the tree do not stir anything either
    rc, info, launches, entries = hop.hop_plan_session_finish(s)
    assert rc == hop.HOP_OK and info["n_launches"] == 1 and len(entries) == n
    assert dt < 0.5, dt
