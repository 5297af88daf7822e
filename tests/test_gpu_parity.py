"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle.

Bit-exact everywhere: integers always, floats because the library evaluates
the same tree order as the oracle.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2002_05814_amd as hop
import workloads

pytestmark = pytest.mark.gpu

ORA_OP = {"sum": oracle.SUM, "min": oracle.MIN, "max": oracle.MAX}
ORA_DT = {"f32": oracle.F32, "bf16": oracle.BF16, "i32": oracle.I32}
ES = workloads.ELEM_BYTES


def dev():
    assert torch.cuda.is_available()
    return torch.device("cuda:0")


def bits(a):
    return a.view(np.uint32) if a.dtype == np.float32 else a


def run_both(w, op, objs=None, order="w", fm="w", check_info=True):
    """One workload through hop_reduce and through the oracle; asserts equality; returns info."""
    objs = workloads.make_objects(w, device=dev()) if objs is None else objs
    order = w.ready_order() if isinstance(order, str) else order
    fm = w.fail_mask() if isinstance(fm, str) else fm
    dst = torch.full_like(objs[0], 77)
    print("case", w.name, w.dtype, op, "bytes", w.object_bytes, "chunk", w.chunk_bytes, "k", w.k, "d", w.tree_degree,
          flush=True)
    rc, info = hop.hop_reduce(dst, objs, w.k, op, w.dtype, w.chunk_bytes, w.tree_degree, order, fm)
    torch.cuda.synchronize()
    d = info["degree_used"] if w.tree_degree == 0 else w.tree_degree
    orc, want, k_eff, n_rep = oracle.reduce([workloads.to_numpy(o) for o in objs], w.k, ORA_OP[op], ORA_DT[w.dtype],
                                            max(1, w.chunk_bytes // ES[w.dtype]), d, order, fm)
    assert rc == orc, (rc, orc)
    if rc >= 0:
        got = workloads.to_numpy(dst)
        assert np.array_equal(bits(got), bits(want)), "mismatch at %s" % np.flatnonzero(bits(got) != bits(want))[:8]
        if check_info:
            assert info["k_eff"] == k_eff and info["n_replaced"] == n_rep
    return rc, info


# ------------------------------------------------------------------ the five workloads, oracle-sized

def test_cfg1_full_size():
    rc, info = run_both(workloads.WORKLOADS[1], "sum")
    assert rc == hop.HOP_OK and info["n_launches"] == 1


def test_cfg2_scaled_ragged():
    # 1 MiB + 12 bytes per object: many tiles, a ragged last chunk and a sub-vector tail
    w = workloads.WORKLOADS[2].scaled((1 << 20) + 12, 64 << 10)
    rc, info = run_both(w, "sum")
    assert rc == hop.HOP_OK and info["k_eff"] == 12


def test_cfg3_scaled_allreduce():
    w = workloads.WORKLOADS[3].scaled(256 << 10, 16 << 10)
    objs = workloads.make_objects(w, device=dev())
    dsts = [torch.full_like(objs[0], -5) for _ in range(w.n_dst)]
    rc, info = hop.hop_allreduce(dsts, objs, w.k, "sum", w.dtype, w.chunk_bytes, w.tree_degree, w.ready_order(), None)
    torch.cuda.synchronize()
    assert rc == hop.HOP_OK and info["k_eff"] == 64
    orc, outs, _, _ = oracle.allreduce([workloads.to_numpy(o) for o in objs], w.n_dst, w.k, oracle.SUM, oracle.I32,
                                       w.chunk_bytes // 4, info["degree_used"], w.ready_order(), None)
    for got, want in zip(dsts, outs):
        assert np.array_equal(workloads.to_numpy(got), want)


def test_cfg4_scaled_failure():
    # 32 bf16 objects of 1 MiB + 6 bytes, 33 chunks; participant 7 fails after its 10th chunk
    w = workloads.WORKLOADS[4].scaled((1 << 20) + 6, 32 << 10)
    rc, info = run_both(w, "sum")
    assert rc == hop.HOP_PARTIAL and info["k_eff"] == 31 and info["n_launches"] == 2
    assert info["chunks_redone"] == 10 * 31


@pytest.mark.parametrize("op", ["max", "sum"])
def test_cfg5_full_size(op):
    rc, info = run_both(workloads.WORKLOADS[5], op)
    assert rc == hop.HOP_OK and info["k_eff"] == 1000 and info["stack_depth"] == 3


# ------------------------------------------------------------------ all dtypes x ops x shapes, with failures

@pytest.mark.parametrize("dtype", ["f32", "bf16", "i32"])
@pytest.mark.parametrize("op", ["sum", "min", "max"])
def test_random_shapes_and_failures(dtype, op):
    rng = np.random.default_rng(1000 + 10 * ["f32", "bf16", "i32"].index(dtype) + ["sum", "min", "max"].index(op))
    base = workloads.WORKLOADS[{"f32": 2, "bf16": 4, "i32": 3}[dtype]]
    for it in range(12):
        n = int(rng.integers(1, 40))
        k = int(rng.integers(1, n + 1))
        d = int(rng.choice([1, 2, 3, 4, 8, 16, n + 3]))
        chunk = 16 * int(rng.integers(1, 300))
        n_elems = int(rng.integers(1, 40000))
        nbytes = n_elems * ES[dtype]
        C = -(-nbytes // chunk)
        w = base.scaled(nbytes, chunk, n=n, k=k, tree_degree=d, order_seed=int(rng.integers(1 << 30)),
                        data_seed=int(rng.integers(1 << 30)), fail={}, name="rand%d" % it)
        fm = None
        if it % 3:
            fm = np.full(n, -1, np.int64)
            bad = rng.random(n) < 0.3
            fm[bad] = rng.integers(0, C + 2, size=int(bad.sum()))
        run_both(w, op, fm=fm)


@pytest.mark.parametrize("d", [1, 2, 16, 64])
def test_every_input_count_up_to_forty(d):
    # chains, binary trees, wide trees and stars over 1..40 inputs: the kernel takes the steps in groups of
    # eight, and groups that consist of plain combines into one level in one go; every count puts the group
    # boundaries elsewhere in the program
    base = workloads.WORKLOADS[2]
    for n in range(1, 41):
        w = base.scaled(200 * 4 + 4, 512, n=n, k=n, tree_degree=d, order_seed=500 + n, data_seed=600 + n, fail={},
                        name="count%d" % n)
        run_both(w, "sum")
    w = workloads.WORKLOADS[4].scaled(200 * 2 + 2, 512, n=37, k=35, tree_degree=d, order_seed=5, data_seed=6, fail={},
                                      name="count_bf16")
    run_both(w, "sum")
    run_both(w, "min")


@pytest.mark.parametrize("dtype", ["f32", "i32", "bf16"])
def test_many_small_objects_take_the_multi_pass_path(dtype):
    # hundreds of inputs, few tiles: programs are cut into passes of independent subtrees (bf16: with fp32 partial results);
    # results must not change by a bit
    rng = np.random.default_rng({"f32": 71, "i32": 72, "bf16": 73}[dtype])
    base = workloads.WORKLOADS[{"f32": 5, "bf16": 4, "i32": 3}[dtype]]
    dist = {"f32": "uniform_pm1", "bf16": "normal_std1", "i32": "randint_pm2p20"}[dtype]
    for it in range(10):
        n = int(rng.integers(64, 700))
        k = int(rng.integers(64, n + 1))
        d = int(rng.choice([2, 3, 4, 8, 16, 32]))
        n_elems = int(rng.integers(1, 3000))
        nbytes = n_elems * ES[dtype]
        chunk = 16 * int(rng.integers(1, 200))
        C = -(-nbytes // chunk)
        w = base.scaled(nbytes, chunk, n=n, k=k, tree_degree=d, order_seed=int(rng.integers(1 << 30)),
                        data_seed=int(rng.integers(1 << 30)), fail={}, name="small%d" % it, dist=dist, n_dst=0)
        fm = None
        if it % 2:
            fm = np.full(n, -1, np.int64)
            bad = rng.random(n) < 0.1
            fm[bad] = rng.integers(0, C + 1, size=int(bad.sum()))
        for op in ("sum", "max"):
            run_both(w, op, fm=fm)
    # thousands of inputs in a binary tree: the program is cut in two rounds (two passes and the top)
    w = base.scaled(256 * ES[dtype], 256 * ES[dtype], n=4000, k=3900, tree_degree=2, order_seed=77, data_seed=78,
                    fail={}, name="small_deep", dist=dist, n_dst=0)
    run_both(w, "sum")
    # objects of a few hundred KiB: still cut (a wave alone would walk 1900 steps), with tens of MiB of partials
    # (bf16: the partial results are 4-byte accumulators, and the steps that read them say so)
    w = base.scaled(300 * 1024 + 4, 1 << 20, n=2000, k=1900, tree_degree=16, order_seed=79, data_seed=80,
                    fail={}, name="small_wide", dist=dist, n_dst=0)
    run_both(w, "sum")
    # the same over chunk runs that neither start nor end at a multiple of 1 KiB (the blocks in which bf16's
    # partial results are laid out), beyond the one-launch form's 64 KiB, and with a ragged last chunk
    w = base.scaled(70 * 1024 * 3 + 2 * ES[dtype], 16 * 4500, n=300, k=290, tree_degree=4, order_seed=81, data_seed=82,
                    fail={}, name="small_chunks", dist=dist, n_dst=0)
    for op in ("sum", "min"):
        run_both(w, op)
    fm = np.full(300, -1, np.int64)
    fm[[5, 77, 200]] = [0, 1, 2]
    run_both(w, "sum", fm=fm)


def takes_the_one_launch_path(w, order=None, fm=None, wide=False):
    """Whether the library evaluates this call's final program as chains in one launch: at least 48 steps
    over at most 64 KiB, the longest path through the chains at most half the program, at most 3072
    workgroup rounds (64-byte columns x rounds of 64 chains), and the values that are alive at one time fit
    the LDS beside the identity value. wide: the same question for the form with 1 KiB columns, which takes
    ranges above 64 KiB up to 768 KiB and whose values are sixteen times as large."""
    _, _, launches, entries = hop.hop_plan_reduce(w.n, w.object_bytes, w.k, w.dtype, w.chunk_bytes, w.tree_degree,
                                                  w.ready_order() if order is None else order, fm)
    final = entries[launches[-1][2]:launches[-1][3]]
    early = w.dtype == "bf16" and w.object_bytes > (32 << 10) and len(final) <= 384      # bf16: wide from 32 KiB for short programs
    if wide:
        if len(final) < 48 or not ((64 << 10) < w.object_bytes <= (768 << 10) or (early and w.object_bytes <= (64 << 10))):
            return False
        src, chains = hop.hop_plan_chains(final, 4)
        if src != hop.HOP_OK:
            return False
        n_pass = 1 + max(p for p, _ in chains)
        critical = sum(max(len(items) for p, items in chains if p == q) for q in range(n_pass))
        read_in = {-it - 1: p for p, items in chains for it in items if it < 0}
        alive = max(sum(1 for g, (p, _) in enumerate(chains) if g in read_in and p <= q <= read_in[g]) for q in range(n_pass))
        return n_pass <= 24 and 2 * critical <= len(final) and alive <= (64 if w.dtype == "bf16" else 128) - 1     # 128 KiB of LDS
    if len(final) < 48 or w.object_bytes > (64 << 10) or early:   # a call without failures is one launch over the object
        return False
    src, chains = hop.hop_plan_chains(final, 4)
    if src != hop.HOP_OK:
        return False
    n_pass = 1 + max(p for p, _ in chains)
    critical = sum(max(len(items) for p, items in chains if p == q) for q in range(n_pass))
    # a chain's value occupies 16 B (bf16: 32 B) x 4 lanes of the workgroup's 64 KiB of LDS from its own pass to
    # the pass that reads it
    read_in = {-it - 1: p for p, items in chains for it in items if it < 0}
    alive = max(sum(1 for g, (p, _) in enumerate(chains) if g in read_in and p <= q <= read_in[g]) for q in range(n_pass))
    # a workgroup has 64 teams: a pass with more chains takes several rounds
    rounds = sum(-(-sum(1 for p, _ in chains if p == q) // 64) for q in range(n_pass))
    columns = -(-w.object_bytes // 64)
    return (n_pass <= 24 and 2 * critical <= len(final) and alive <= (512 if w.dtype == "bf16" else 1024) - 1
            and columns * rounds <= 3072)


CHAIN_CASES = [
    # dtype, n, k, d, object bytes, chunk bytes
    ("f32", 1024, 1000, 16, 4096, 4096),             # workload 5
    ("f32", 300, 300, 4, 4, 64),                     # one element: only the workgroup for the ragged end
    ("f32", 200, 190, 8, 12, 64),
    ("bf16", 500, 500, 16, 14, 64),                  # seven elements behind no vector at all: two workgroups of four lanes
    ("bf16", 500, 400, 8, 16, 16),                   # exactly one vector
    ("i32", 120, 120, 2, 252, 1024),                 # three columns, three vectors of a fourth and three elements; a binary tree
    ("f32", 300, 280, 3, 256 + 4, 4096),             # four columns and one element
    ("bf16", 900, 900, 32, 4096 + 2 * 5, 8192),
    ("i32", 1000, 1000, 16, 65536 - 4, 16384),       # the largest range: 1024 columns less an element
    ("f32", 2000, 2000, 16, 1000 * 4, 1024),         # four chunks, the last one ragged; more chains than teams
    ("bf16", 1500, 1400, 40, 30 * 2, 4096),          # nodes with 40 children: folds longer than a record, cut in two
    ("f32", 100, 100, 2, 8192, 2048),                # a binary tree: five passes
    ("f32", 5000, 5000, 2, 512, 512),                # a binary tree on 5000: too many chains, the older path
    ("f32", 1024, 1000, 16, 131072, 65536),          # workload 5 with larger objects: the older path
    ("i32", 48, 48, 4, 640, 4096),                   # the shortest program that takes the path
    ("f32", 150, 150, 4, 64 * 45 + 12, 4096),        # 45 columns: one whole block of 32 in die order, 13 in plain order
    ("i32", 200, 180, 16, 6400, 2560),               # chunks of 40, 40 and 20 columns
]


@pytest.mark.parametrize("dtype,n,k,d,nbytes,chunk", CHAIN_CASES)
def test_long_programs_over_small_objects_in_one_launch(dtype, n, k, d, nbytes, chunk):
    base = workloads.WORKLOADS[{"f32": 5, "bf16": 4, "i32": 3}[dtype]]
    dist = {"f32": "uniform_pm1", "bf16": "normal_std1", "i32": "randint_pm2p20"}[dtype]
    w = base.scaled(nbytes, chunk, n=n, k=k, tree_degree=d, order_seed=n + d, data_seed=k + nbytes, fail={},
                    name="chains_%s_%d" % (dtype, n), dist=dist, n_dst=0)
    assert takes_the_one_launch_path(w) == (n != 5000 and nbytes != 131072)
    objs = workloads.make_objects(w, device=dev())
    for op in ("sum", "min", "max"):
        rc, info = run_both(w, op, objs=objs)
        assert rc == hop.HOP_OK and info["n_launches"] == 1
    # with failures before and in the middle of the stream (holes, replacements, repairs of produced chunks)
    rng = np.random.default_rng(n * 7 + d)
    fm = np.full(n, -1, np.int64)
    bad = rng.random(n) < 0.08
    fm[bad] = rng.integers(0, w.n_chunks + 1, size=int(bad.sum()))
    run_both(w, "sum", objs=objs, fm=fm)
    # all-reduce: the copy to the other destinations follows the one launch
    dsts = [torch.full_like(objs[0], 3) for _ in range(3)]
    rc, info = hop.hop_allreduce(dsts, objs, w.k, "sum", w.dtype, w.chunk_bytes, w.tree_degree, w.ready_order(), None)
    torch.cuda.synchronize()
    orc, outs, _, _ = oracle.allreduce([workloads.to_numpy(o) for o in objs], 3, w.k, oracle.SUM, ORA_DT[dtype],
                                       max(1, w.chunk_bytes // ES[dtype]), d, w.ready_order(), None)
    assert rc == orc == hop.HOP_OK
    for got, want in zip(dsts, outs):
        assert np.array_equal(bits(workloads.to_numpy(got)), bits(want))


WIDE_CHAIN_CASES = [
    # dtype, n, k, d, object bytes, chunk bytes, takes the wide form
    ("f32", 200, 190, 16, 256 * 1024 + 12, 1 << 20, True),        # 257 columns of 1 KiB less most of the last, and three elements
    ("i32", 1000, 990, 16, 100 * 1024, 1 << 20, True),
    ("f32", 300, 280, 2, 72000 * 3 - 40, 72000, True),            # a binary tree: 70 values alive at a time, more than 64 KiB of LDS
    ("f32", 300, 280, 8, 72000 * 3 - 40, 72000, True),            # with failures: chunk runs of 72000 bytes that start anywhere
    ("bf16", 128, 128, 8, 200 * 1024 + 2, 1 << 20, True),         # values of 2 KiB: 31 at a time
    ("bf16", 1000, 1000, 16, 128 * 1024, 1 << 20, True),          # 59 values of 2 KiB alive at a time
    ("bf16", 2000, 2000, 16, 96 * 1024, 1 << 20, False),          # more values alive than bf16 has room for: cut into sub-programs
    ("f32", 60, 60, 4, 300 * 1024, 1 << 20, True),                # a short program
    ("bf16", 200, 200, 16, 48 * 1024 + 6, 1 << 20, True),         # bf16 takes the wide form from 32 KiB for short programs
    ("i32", 100, 100, 4, 768 * 1024, 1 << 20, True),              # the longest range
    ("f32", 4000, 4000, 16, 80 * 1024, 1 << 20, False),           # more values alive than fit: cut into sub-programs
]


@pytest.mark.parametrize("dtype,n,k,d,nbytes,chunk,wide", WIDE_CHAIN_CASES)
def test_long_programs_over_medium_objects_in_one_launch_of_wide_columns(dtype, n, k, d, nbytes, chunk, wide):
    base = workloads.WORKLOADS[{"f32": 5, "bf16": 4, "i32": 3}[dtype]]
    dist = {"f32": "uniform_pm1", "bf16": "normal_std1", "i32": "randint_pm2p20"}[dtype]
    w = base.scaled(nbytes, chunk, n=n, k=k, tree_degree=d, order_seed=n + d + 1, data_seed=k + nbytes + 1, fail={},
                    name="wide_%s_%d" % (dtype, n), dist=dist, n_dst=0)
    assert takes_the_one_launch_path(w, wide=True) == wide
    objs = workloads.make_objects(w, device=dev())
    for op in ("sum", "min", "max"):
        rc, info = run_both(w, op, objs=objs)
        assert rc == hop.HOP_OK and info["n_launches"] == 1
    # failures before and in the middle of the stream: launches over runs of chunks, holes, replacements, repairs
    rng = np.random.default_rng(n * 5 + d)
    fm = np.full(n, -1, np.int64)
    bad = rng.random(n) < 0.05
    fm[bad] = rng.integers(0, w.n_chunks + 1, size=int(bad.sum()))
    run_both(w, "sum", objs=objs, fm=fm)
    # all-reduce: the copy to the other destinations follows the one launch
    dsts = [torch.full_like(objs[0], 3) for _ in range(2)]
    rc, info = hop.hop_allreduce(dsts, objs, w.k, "max", w.dtype, w.chunk_bytes, w.tree_degree, w.ready_order(), None)
    torch.cuda.synchronize()
    orc, outs, _, _ = oracle.allreduce([workloads.to_numpy(o) for o in objs], 2, w.k, oracle.MAX, ORA_DT[dtype],
                                       max(1, w.chunk_bytes // ES[dtype]), d, w.ready_order(), None)
    assert rc == orc == hop.HOP_OK
    for got, want in zip(dsts, outs):
        assert np.array_equal(bits(workloads.to_numpy(got)), bits(want))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_one_launch_path_with_specials_and_sources_at_odd_alignment(dtype):
    # NaNs, infinities, signed zeros and denormals through the chains' folds and their values in LDS; the
    # objects are views 16 bytes into their allocations (bf16: the upper halves of the same fp32 patterns)
    es = ES[dtype]
    n, nbytes = 400, 1000 * es
    w = workloads.WORKLOADS[{"f32": 5, "bf16": 4}[dtype]].scaled(nbytes, 4096, n=n, k=n, tree_degree=8, order_seed=3,
                                                                 data_seed=4, fail={}, name="chains_specials", n_dst=0)
    assert takes_the_one_launch_path(w)
    rng = np.random.default_rng(12)
    # every element position has one theme, so that two different NaNs never meet (which of them a sum
    # returns is not defined): +inf among finite values, -inf, both (the sum generates a NaN), one quiet NaN
    # pattern, zeros of both signs only, denormals only, large values that overflow, plain values
    E = nbytes // es
    theme = rng.integers(0, 8, size=E)
    qnan = np.array([0x7fc01234], np.uint32).view(np.float32)[0]
    tdt = {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]
    backing = [torch.zeros(E + 16 // es * 2, dtype=tdt, device=dev()) for _ in range(n)]
    objs = []
    for b in backing:
        host = (rng.standard_normal(E) * 1e-3).astype(np.float32)
        hit = rng.random(E) < 0.03
        host[hit & (theme == 0)] = np.inf
        host[hit & (theme == 1)] = -np.inf
        both = hit & (theme == 2)
        host[both] = np.where(rng.random(int(both.sum())) < 0.5, np.inf, -np.inf).astype(np.float32)
        host[hit & (theme == 3)] = qnan
        zeros = theme == 4
        host[zeros] = np.where(rng.random(int(zeros.sum())) < 0.5, 0.0, -0.0).astype(np.float32)
        den = theme == 5
        host[den] = (rng.standard_normal(int(den.sum())) * 1e-42).astype(np.float32)
        big = theme == 6
        host[big] = (rng.standard_normal(int(big.sum())) * 3e37).astype(np.float32)
        o = b[16 // es:16 // es + E]
        if dtype == "bf16":
            host = (host.view(np.uint32) >> 16).astype(np.uint16)       # truncated: themes and specials survive
        o.copy_(workloads.from_numpy(host, dtype))
        objs.append(o)
    for op in ("sum", "min", "max"):
        run_both(w, op, objs=objs)


def test_infinities_and_nans_come_out_as_in_the_oracle():
    # at most one NaN meets any element position (which of two NaN payloads an addition keeps is not
    # fixed by the C the oracle is written in): inf - inf, inf + finite, a quiet NaN with a payload, a
    # signalling NaN that meets a number, a signalling NaN that meets only zeros, NaNs in min and max
    d = dev()
    E = 64
    vals = [np.zeros(E, np.float32) for _ in range(4)]
    qnan = np.array([0x7fc01234], np.uint32).view(np.float32)[0]
    snan = np.array([0x7f801234], np.uint32).view(np.float32)[0]
    vals[0][0], vals[1][0] = np.inf, -np.inf
    vals[0][1], vals[2][1] = np.inf, 1.0
    vals[1][2], vals[2][2] = qnan, 2.0
    vals[3][3], vals[0][3] = snan, 1.0
    vals[2][5] = snan
    vals[3][6], vals[1][6] = -np.inf, -np.inf
    objs = [workloads.from_numpy(x, "f32", d) for x in vals]
    for op in ("sum", "max", "min"):
        for deg in (1, 2, 4):
            dst = torch.zeros(E, device=d)
            rc, info = hop.hop_reduce(dst, objs, 4, op, "f32", 256, deg, None, None)
            torch.cuda.synchronize()
            orc, want, _, _ = oracle.reduce(vals, 4, ORA_OP[op], oracle.F32, 64, deg, None, None)
            assert rc == orc == hop.HOP_OK
            assert np.array_equal(bits(workloads.to_numpy(dst)), bits(want)), (op, deg)
    # a reduce of one object is a copy, signalling NaNs included
    dst = torch.zeros(E, device=d)
    rc, _ = hop.hop_reduce(dst, objs[3:4], 1, "sum", "f32", 256, 2, None, None)
    torch.cuda.synchronize()
    assert rc == hop.HOP_OK and np.array_equal(bits(workloads.to_numpy(dst)), bits(vals[3]))
    # bf16: the same cases as 16-bit patterns, plus sums that overflow to infinity and a sum whose fp32
    # value rounds up into the next bf16 binade at the one final rounding
    b = [np.zeros(E, np.uint16) for _ in range(4)]
    b[0][0], b[1][0] = 0x7f80, 0xff80                      # inf + -inf
    b[0][1], b[2][1] = 0x7f80, 0x3f80                      # inf + 1
    b[1][2], b[2][2] = 0x7fc1, 0x4000                      # quiet NaN with a payload + 2
    b[3][3], b[0][3] = 0x7f81, 0x3f80                      # signalling NaN + 1
    b[2][5] = 0x7f81                                       # signalling NaN + zeros
    b[0][6], b[1][6], b[2][6] = 0x7f7f, 0x7f7f, 0x7f7f     # three times the largest finite value
    b[0][7], b[1][7] = 0x3fff, 0x3b80                      # 1.9921875 + 2^-8: a tie at bf16 precision
    bobjs = [workloads.from_numpy(x, "bf16", d) for x in b]
    for op in ("sum", "max", "min"):
        for deg in (1, 2, 4):
            dst = torch.zeros(E, dtype=torch.bfloat16, device=d)
            rc, info = hop.hop_reduce(dst, bobjs, 4, op, "bf16", 128, deg, None, None)
            torch.cuda.synchronize()
            orc, want, _, _ = oracle.reduce(b, 4, ORA_OP[op], oracle.BF16, 64, deg, None, None)
            assert rc == orc == hop.HOP_OK
            assert np.array_equal(workloads.to_numpy(dst), want), (op, deg)


def test_denormals_and_signed_zeros_are_preserved():
    w = workloads.WORKLOADS[1].scaled(4096 * 4, 1024, n=4, k=4)
    rng = np.random.default_rng(5)
    vals = []
    for i in range(4):
        v = (rng.standard_normal(4096) * 1e-41).astype(np.float32)      # denormal range
        v[::7] = 0.0
        v[3::7] = -0.0
        vals.append(v)
    objs = [workloads.from_numpy(v, "f32", dev()) for v in vals]
    for op in ("sum", "min", "max"):
        run_both(w, op, objs=objs)


def test_bf16_every_pattern_rounds_like_the_oracle():
    # object 0 holds every finite bf16 pattern; the others add values that land on ties and near-ties
    h = np.arange(1 << 16, dtype=np.uint16)
    f = (h.astype(np.uint32) << 16).view(np.float32)
    h = h[np.isfinite(f)]
    E = h.size
    w = workloads.WORKLOADS[4].scaled(E * 2, 4096, n=3, k=3, tree_degree=2, fail={})
    for addend in (2.0 ** -8, 2.0 ** -9, 3 * 2.0 ** -9, 1.0, -2.0 ** -8, 1e-3, 255.0):
        a = torch.full((E,), addend, dtype=torch.float32).to(torch.bfloat16)
        b = torch.full((E,), addend * 2.0 ** -8, dtype=torch.float32).to(torch.bfloat16)
        objs = [workloads.from_numpy(h, "bf16", dev()), a.to(dev()), b.to(dev())]
        run_both(w, "sum", objs=objs, order=None, fm=None)


# ------------------------------------------------------------------ edges and errors

def test_tiny_and_empty_objects():
    for dtype in ("f32", "bf16", "i32"):
        for n_elems in (0, 1, 2, 3, 4, 5, 7, 8, 9):
            w = workloads.WORKLOADS[1].scaled(n_elems * ES[dtype], 16, n=5, k=3, dtype=dtype,
                                              dist={"f32": "uniform_pm1", "bf16": "normal_std1",
                                                    "i32": "randint_pm2p20"}[dtype])
            if n_elems == 0:
                objs = [torch.zeros(4, dtype=workloads.TORCH_DTYPE[dtype], device=dev()) for _ in range(5)]
                dst = torch.full_like(objs[0], 9)
                rc, info = hop.hop_reduce(dst, objs, 3, "sum", dtype, 16, 2, None, None, object_bytes=0)
                torch.cuda.synchronize()
                assert rc == hop.HOP_OK and info["k_eff"] == 3
                assert torch.all(dst == 9)                  # nothing written
            else:
                run_both(w, "sum", order=None)


def test_k1_and_n1():
    w = workloads.WORKLOADS[1].scaled(4000, 1024, n=1, k=1)
    run_both(w, "sum", order=None)
    w = workloads.WORKLOADS[1].scaled(4000, 1024, n=6, k=1)
    run_both(w, "max", order=np.array([4, 2, 0, 1, 3, 5], np.int32))


def test_errors():
    d = dev()
    objs = [torch.zeros(1024, device=d) for _ in range(4)]
    dst = torch.zeros(1024, device=d)
    R = hop.hop_reduce
    assert R(dst, objs, 5, "sum", "f32", 1024, 2)[0] == hop.HOP_ERR_INVALID
    assert R(dst, objs, 2, "sum", "f32", 100, 2)[0] == hop.HOP_ERR_INVALID
    assert R(dst, objs, 2, "sum", "f32", 1024, 2, ready_order=[0, 0, 1, 2])[0] == hop.HOP_ERR_INVALID
    assert R(dst, objs, 2, "sum", "f32", 1024, 2, fail_mask=[0, 0, 0, 0])[0] == hop.HOP_ERR_NO_SURVIVOR
    assert R(objs[1], objs, 2, "sum", "f32", 1024, 2)[0] == hop.HOP_ERR_INVALID          # result over a source
    mis = [objs[0], objs[1][1:], objs[2], objs[3]]
    assert R(dst, mis, 2, "sum", "f32", 1024, 2, object_bytes=4000)[0] == hop.HOP_ERR_ALIGN
    assert R(dst[1:], objs, 2, "sum", "f32", 1024, 2, object_bytes=4000)[0] == hop.HOP_ERR_ALIGN
    assert hop.hop_broadcast([dst[1:]], objs[0], 1024, object_bytes=4000) == hop.HOP_ERR_ALIGN
    assert hop.hop_broadcast([dst], dst, 1024) == hop.HOP_ERR_INVALID
    # destinations that overlap each other (the same buffer twice, or shifted by less than an object)
    big = torch.zeros(2048, device=d)
    assert hop.hop_broadcast([big[:1024], big[:1024]], objs[0], 1024) == hop.HOP_ERR_INVALID
    assert hop.hop_broadcast([big[:1024], big[512:1536]], objs[0], 1024) == hop.HOP_ERR_INVALID
    assert hop.hop_allreduce([big[512:1536], big[:1024]], objs, 2, "sum", "f32", 1024, 2)[0] == hop.HOP_ERR_INVALID
    assert hop.hop_allreduce([big[:1024], big[1024:]], objs, 2, "sum", "f32", 1024, 2)[0] == hop.HOP_OK
    torch.cuda.synchronize()


# ------------------------------------------------------------------ broadcast

def test_broadcast_paper_object_and_ragged_sizes():
    d = dev()
    src = torch.tensor([5, 1, 0], dtype=torch.int32, device=d)            # the array of figure 4
    buf = [torch.zeros(4, dtype=torch.int32, device=d) for _ in range(3)]
    assert hop.hop_broadcast(buf, src, 16, object_bytes=12) == hop.HOP_OK
    torch.cuda.synchronize()
    for b in buf:
        assert b.tolist() == [5, 1, 0, 0]
    rng = np.random.default_rng(2)
    for nbytes in (1, 15, 16, 17, 4095, 1 << 20, (1 << 20) + 5):
        blob = rng.integers(0, 256, size=nbytes, dtype=np.uint8)
        s = torch.from_numpy(blob).to(d)
        outs = [torch.zeros(nbytes + 3, dtype=torch.uint8, device=d) for _ in range(5)]
        assert hop.hop_broadcast(outs, s, 4096, object_bytes=nbytes) == hop.HOP_OK
        torch.cuda.synchronize()
        want = oracle.broadcast(blob, 5)
        for o, wv in zip(outs, want):
            assert np.array_equal(o[:nbytes].cpu().numpy(), wv) and int(o[nbytes:].sum()) == 0
    assert hop.hop_broadcast([], src, 16) == hop.HOP_OK


def test_broadcast_over_several_spans_with_a_ragged_end():
    # the copy to several destinations walks the source in 16 MiB spans, destination by destination:
    # sizes around one, two and three spans, a last tile that is not full, bytes beyond the last vector
    d = dev()
    rng = np.random.default_rng(77)
    span = 16 << 20
    for nbytes, n_dst in ((span, 2), (span + 16, 3), (2 * span - 4096 + 48 + 7, 9), (3 * span + 5, 2), (span - 3, 1),
                          ((41 << 20) + 5 * 1024 + 21, 1)):        # long one-to-one copy: pieces 64 KiB apart, a ragged last group
        blob = rng.integers(0, 256, size=nbytes, dtype=np.uint8)
        s = torch.from_numpy(blob).to(d)
        outs = [torch.zeros(nbytes + 16, dtype=torch.uint8, device=d) for _ in range(n_dst)]
        assert hop.hop_broadcast(outs, s, 1 << 20, object_bytes=nbytes) == hop.HOP_OK
        torch.cuda.synchronize()
        for o in outs:
            assert torch.equal(o[:nbytes], s) and int(o[nbytes:].sum()) == 0, (nbytes, n_dst)


@pytest.mark.parametrize("nbytes,n_dst", [((41 << 20) + 5 * 1024 + 21, 1), ((17 << 20) + 333, 3), (70001, 4), (100, 2), (9, 3)])
def test_broadcast_to_destinations_that_are_only_16_byte_aligned(nbytes, n_dst):
    # destinations 16..112 bytes past a 128-byte boundary (the copy kernels start their stores at a boundary
    # of most destinations and skip what lies in front), the source 32 bytes past one
    d = dev()
    rng = np.random.default_rng(nbytes)
    slot = (nbytes + 1023) // 1024 * 1024 + 1024
    pool = torch.zeros((n_dst + 1) * slot, dtype=torch.uint8, device=d)
    assert pool.data_ptr() % 128 == 0
    src = pool[32:32 + nbytes]
    src.copy_(torch.from_numpy(rng.integers(1, 256, size=nbytes, dtype=np.uint8)).to(d))
    res = [16, 16, 80, 112][:n_dst]
    outs = [pool[(j + 1) * slot + res[j]:(j + 1) * slot + res[j] + nbytes] for j in range(n_dst)]
    assert hop.hop_broadcast(outs, src, 1 << 20, object_bytes=nbytes) == hop.HOP_OK
    torch.cuda.synchronize()
    for j, o in enumerate(outs):
        assert torch.equal(o, src), j
        lo = (j + 1) * slot
        assert int(pool[lo:lo + res[j]].sum()) == 0 and int(pool[lo + res[j] + nbytes:lo + slot].sum()) == 0, j


def test_copies_see_what_was_written_just_before():
    # the copy to several destinations reads its source through the caches, and reads it again per
    # destination: a source rewritten between two calls (by the reduce kernel, by another library) must come
    # out new, in every destination, every time
    d = dev()
    E = (4 << 20) + 1024 + 12
    dsts = [torch.zeros(E, dtype=torch.int32, device=d) for _ in range(5)]
    objs = [torch.zeros(E, dtype=torch.int32, device=d) for _ in range(8)]
    g = torch.Generator(device=d)
    g.manual_seed(99)
    for rnd in range(4):
        for o in objs:
            o.random_(-1000, 1000, generator=g)
        rc, _ = hop.hop_allreduce(dsts, objs, 8, "sum", "i32", 1 << 20, 2, None, None)
        assert rc == hop.HOP_OK
        want = torch.zeros_like(objs[0])
        for o in objs:
            want += o
        for t in dsts:
            assert torch.equal(t, want), rnd
    src = torch.zeros(E, dtype=torch.int32, device=d)
    outs = [torch.zeros(E, dtype=torch.int32, device=d) for _ in range(6)]
    for rnd in range(4):
        src.random_(-1000, 1000, generator=g)
        assert hop.hop_broadcast(outs, src, 1 << 20) == hop.HOP_OK
        for t in outs:
            assert torch.equal(t, src), rnd


def test_receiver_driven_broadcast_chains_and_survives_a_lost_copy():
    d = dev()
    rng = np.random.default_rng(21)
    C, chunk = 7, 4096
    nbytes = (C - 1) * chunk + 1000
    blob = rng.integers(0, 256, size=nbytes, dtype=np.uint8)
    src = torch.from_numpy(blob).to(d)
    bufs = [torch.zeros(nbytes, dtype=torch.uint8, device=d) for _ in range(6)]
    rc, b = hop.hop_bcast_begin(src, nbytes, chunk)
    assert rc == hop.HOP_OK
    assert hop.hop_bcast_source_ready(b, 3) == hop.HOP_OK              # the original is still being written
    ids = []
    for i in range(3):
        rid, s = hop.hop_bcast_join(b, bufs[i])
        ids.append(rid)
        assert hop.hop_bcast_step(b, 1) == hop.HOP_OK
    assert [hop.hop_bcast_sender(b, r) for r in ids] == [0, 1, 2]      # a chain through partial copies
    assert hop.hop_bcast_fail(b, ids[1]) == hop.HOP_OK                 # the middle of the chain is lost
    assert hop.hop_bcast_source_ready(b, C) == hop.HOP_OK
    for i in range(3, 6):
        rid, s = hop.hop_bcast_join(b, bufs[i])
        ids.append(rid)
        hop.hop_bcast_step(b, 2)
    assert hop.hop_bcast_join(b, bufs[0])[0] == hop.HOP_ERR_INVALID    # a buffer cannot be two copies
    rc, info, log = hop.hop_bcast_finish(b)
    torch.cuda.synchronize()
    assert rc == hop.HOP_OK and info["n_complete"] == 5 and info["n_failed"] == 1 and info["n_resumed"] == 1
    want = oracle.broadcast(blob, 1)[0]
    for i, buf in enumerate(bufs):
        if i != 1:
            assert np.array_equal(buf.cpu().numpy(), want), i
    assert info["chunks_copied"] == sum(c1 - c0 for _, _, c0, c1 in log)


# ------------------------------------------------------------------ event-level sessions

def session_replay(objs, dst, k, op, dtype, chunk, d, order, fm, C, fine, eager=0, workspace=None, stream=None):
    """Drives the session API with the same timeline hop_reduce replays, either in bulk
    (per failure step) or chunk by chunk."""
    rc, s = hop.hop_session_begin(dst, objs, k, op, dtype, chunk, d, stream=stream)
    assert rc == hop.HOP_OK
    if workspace is not None:
        assert hop.hop_session_set_workspace(s, workspace) == hop.HOP_OK
    assert hop.hop_session_set_eager(s, eager) == hop.HOP_OK
    n = len(objs)
    limit = [C if (fm is None or fm[i] < 0 or fm[i] >= C) else int(fm[i]) for i in range(n)]
    arrival = [int(i) for i in order if limit[i] > 0]
    for i in arrival:
        assert hop.hop_session_ready(s, i, 0) == hop.HOP_OK
    alive = set(arrival)
    steps = range(1, C + 1) if fine else sorted({limit[i] for i in arrival if limit[i] < C} | {C})
    prev = 0
    for step in steps:
        for i in arrival:
            if i in alive and min(step, limit[i]) > min(prev, limit[i]):
                assert hop.hop_session_ready(s, i, min(step, limit[i])) == hop.HOP_OK
        for i in arrival:
            if i in alive and limit[i] == step and step < C:
                assert hop.hop_session_fail(s, i) == hop.HOP_OK
                alive.discard(i)
        prev = step
    return hop.hop_session_finish(s)


@pytest.mark.parametrize("fine", [False, True])
def test_session_events_match_oracle(fine):
    rng = np.random.default_rng(31 + fine)
    for it in range(10):
        n = int(rng.integers(2, 20))
        k = int(rng.integers(1, n + 1))
        d = int(rng.choice([1, 2, 4, n]))
        chunk, C = 1024, int(rng.integers(1, 9))
        n_elems = (C - 1) * 256 + int(rng.integers(1, 257))
        order = rng.permutation(n).astype(np.int32)
        fm = np.full(n, -1, np.int64)
        bad = rng.random(n) < 0.3
        fm[bad] = rng.integers(0, C + 1, size=int(bad.sum()))
        vals = [rng.standard_normal(n_elems).astype(np.float32) for _ in range(n)]
        objs = [workloads.from_numpy(v, "f32", dev()) for v in vals]
        dst = torch.zeros(n_elems, device=dev())
        print("session case", it, n, k, d, C, fine, flush=True)
        rc, info = session_replay(objs, dst, k, "sum", "f32", chunk, d, order, fm, C, fine)
        torch.cuda.synchronize()
        orc, want, k_eff, n_rep = oracle.reduce(vals, k, oracle.SUM, oracle.F32, 256, d, order, fm)
        assert rc == orc
        if rc >= 0:
            assert np.array_equal(bits(workloads.to_numpy(dst)), bits(want))
            assert info["k_eff"] == k_eff
            if fine and not bad.any() and C > 1:
                assert info["n_launches"] == C          # one launch per chunk as each becomes complete


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_session_events_over_hundreds_of_small_objects(dtype):
    # the event-level API over many small objects: every launch covers one or a few chunks of at most a few
    # KiB with a program of hundreds of steps (the one-launch form), and every failure changes the program
    rng = np.random.default_rng({"f32": 61, "bf16": 62}[dtype])
    base = workloads.WORKLOADS[{"f32": 5, "bf16": 4}[dtype]]
    es = ES[dtype]
    for it in range(6):
        n = int(rng.integers(100, 400))
        k = int(rng.integers(60, n + 1))
        d = int(rng.choice([3, 4, 8, 16]))
        C = int(rng.integers(2, 6))
        chunk = 16 * int(rng.integers(4, 130))
        nbytes = (C - 1) * chunk + es * int(rng.integers(1, chunk // es + 1))
        w = base.scaled(nbytes, chunk, n=n, k=k, tree_degree=d, order_seed=int(rng.integers(1 << 30)),
                        data_seed=int(rng.integers(1 << 30)), fail={}, name="many%d" % it, n_dst=0,
                        dist={"f32": "uniform_pm1", "bf16": "normal_std1"}[dtype])
        objs = workloads.make_objects(w, device=dev())
        order = w.ready_order()
        fm = np.full(n, -1, np.int64)
        bad = rng.random(n) < 0.05
        fm[bad] = rng.integers(0, C + 1, size=int(bad.sum()))
        dst = torch.full_like(objs[0], 9)
        fine = bool(it % 2)
        print("many-objects session", dtype, it, n, k, d, C, nbytes, fine, flush=True)
        rc, info = session_replay(objs, dst, k, "sum", dtype, chunk, d, order, fm, C, fine)
        torch.cuda.synchronize()
        orc, want, k_eff, n_rep = oracle.reduce([workloads.to_numpy(o) for o in objs], k, oracle.SUM, ORA_DT[dtype],
                                                chunk // es, d, order, fm)
        assert rc == orc
        if rc >= 0:
            assert np.array_equal(bits(workloads.to_numpy(dst)), bits(want))
            assert info["k_eff"] == k_eff and info["n_replaced"] == n_rep


@pytest.mark.parametrize("dtype", ["f32", "bf16", "i32"])
def test_session_eager_segments_match_oracle(dtype):
    # objects arrive whole, one after the other (object-by-object timeline), some failing part-way:
    # with the eager policy every arrival is folded into saved accumulators at once; the bits must
    # equal the fused evaluation's and the oracle's
    rng = np.random.default_rng({"f32": 41, "bf16": 42, "i32": 43}[dtype])
    base = workloads.WORKLOADS[{"f32": 2, "bf16": 4, "i32": 3}[dtype]]
    es = ES[dtype]
    for it in range(8):
        n = int(rng.integers(2, 24))
        k = int(rng.integers(1, n + 1))
        d = int(rng.choice([1, 2, 3, 8]))
        C = int(rng.integers(2, 7))
        chunk = 16 * int(rng.integers(8, 300))
        nbytes = (C - 1) * chunk + es * int(rng.integers(1, chunk // es + 1))
        w = base.scaled(nbytes, chunk, n=n, k=k, tree_degree=d, order_seed=int(rng.integers(1 << 30)),
                        data_seed=int(rng.integers(1 << 30)), fail={}, name="eager%d" % it, n_dst=0)
        objs = workloads.make_objects(w, device=dev())
        order = w.ready_order()
        fm = np.full(n, -1, np.int64)
        bad = rng.random(n) < 0.25
        fm[bad] = rng.integers(1, C, size=int(bad.sum()))
        eager = int(rng.integers(1, 4))
        print("eager case", dtype, it, n, k, d, C, nbytes, eager, flush=True)
        dst = torch.full_like(objs[0], 3)
        rc, s = hop.hop_session_begin(dst, objs, k, "sum", dtype, chunk, d)
        assert rc == hop.HOP_OK and hop.hop_session_set_eager(s, eager) == hop.HOP_OK
        model_slots, pool, dead = [], [], set()
        for i in order:                              # object-major: deliver, then (maybe) fail
            i = int(i)
            c = C if fm[i] < 0 else int(fm[i])
            assert hop.hop_session_ready(s, i, c) == hop.HOP_OK
            if len(model_slots) < k and None not in model_slots:
                model_slots.append(i)
            elif None in model_slots:
                model_slots[model_slots.index(None)] = i
            else:
                pool.append(i)
            if fm[i] >= 0:
                assert hop.hop_session_fail(s, i) == hop.HOP_OK
                dead.add(i)
                if i in model_slots:
                    pool = [p for p in pool if p not in dead]
                    model_slots[model_slots.index(i)] = pool.pop(0) if pool else None
                else:
                    pool = [p for p in pool if p not in dead]
        rc, info = hop.hop_session_finish(s)
        torch.cuda.synchronize()
        slots = model_slots + [None] * (k - len(model_slots))
        live = [o for o in slots if o is not None]
        if not live:
            assert rc == hop.HOP_ERR_NO_SURVIVOR
            continue
        # the oracle's value for this placement: holes are objects that arrive and fail with nobody left
        host = [workloads.to_numpy(o) for o in objs]
        spare = [j for j in range(n) if j not in live]
        o_order, o_fm = [], np.zeros(n, np.int64)
        for o in slots:
            if o is None:
                o = spare.pop()
                o_fm[o] = 1
            else:
                o_fm[o] = -1
            o_order.append(o)
        o_order += spare
        orc, want, k_eff, _ = oracle.reduce(host, k, oracle.SUM, ORA_DT[dtype], chunk // es, d,
                                            np.array(o_order, np.int32), o_fm)
        assert rc == orc and info["k_eff"] == k_eff == len(live)
        assert np.array_equal(bits(workloads.to_numpy(dst)), bits(want))
        assert info["n_launches"] >= 1


def test_session_late_arrival_fills_the_hole_and_unfinished_objects_count_as_failed():
    d = dev()
    rng = np.random.default_rng(3)
    vals = [rng.standard_normal(1024).astype(np.float32) for _ in range(4)]
    objs = [workloads.from_numpy(v, "f32", d) for v in vals]
    dst = torch.zeros(1024, device=d)
    rc, s = hop.hop_session_begin(dst, objs, 3, "sum", "f32", 1024, 2)          # 4 chunks
    for i in (0, 1, 2):
        assert hop.hop_session_ready(s, i, 2) == hop.HOP_OK
    assert hop.hop_session_fail(s, 1) == hop.HOP_OK                              # nobody is waiting: position 1 is empty
    assert hop.hop_session_ready(s, 1, 3) == hop.HOP_ERR_INVALID                 # a failed object cannot come back under the same id
    assert hop.hop_session_ready(s, 3, 4) == hop.HOP_OK                          # late arrival takes position 1
    assert hop.hop_session_ready(s, 0, 4) == hop.HOP_OK
    assert hop.hop_session_ready(s, 0, 3) == hop.HOP_ERR_INVALID                 # counts never decrease
    assert hop.hop_session_ready(s, 2, 4) == hop.HOP_OK
    rc, info = hop.hop_session_finish(s)
    torch.cuda.synchronize()
    assert rc == hop.HOP_OK and info["k_eff"] == 3 and info["n_replaced"] == 1
    _, want, _, _ = oracle.reduce(vals, 3, oracle.SUM, oracle.F32, 256, 2, np.array([0, 3, 2, 1], np.int32), None)
    assert np.array_equal(bits(workloads.to_numpy(dst)), bits(want))
    # object 2 never finishes: at the end it counts as failed
    rc, s = hop.hop_session_begin(dst, objs, 3, "sum", "f32", 1024, 2)
    for i, c in ((0, 4), (1, 4), (2, 1)):
        assert hop.hop_session_ready(s, i, c) == hop.HOP_OK
    rc, info = hop.hop_session_finish(s)
    torch.cuda.synchronize()
    assert rc == hop.HOP_PARTIAL and info["k_eff"] == 2
    fm = np.array([-1, -1, 1, 0], np.int64)
    _, want, _, _ = oracle.reduce(vals, 3, oracle.SUM, oracle.F32, 256, 2, None, fm)
    assert np.array_equal(bits(workloads.to_numpy(dst)), bits(want))


def test_composed_reduce_streams_one_result_into_the_next():
    # paper section 3.4.2: the output of one Reduce is an input of another; as soon as leading chunks
    # of the first result are final they are reported ready to the second session (same stream)
    d = dev()
    rng = np.random.default_rng(12)
    C, ce = 5, 512
    E = (C - 1) * ce + 100
    a_vals = [rng.standard_normal(E).astype(np.float32) for _ in range(4)]
    b_vals = [rng.standard_normal(E).astype(np.float32) for _ in range(2)]
    a_objs = [workloads.from_numpy(v, "f32", d) for v in a_vals]
    b_objs = [workloads.from_numpy(v, "f32", d) for v in b_vals]
    mid = torch.zeros(E, device=d)
    out = torch.zeros(E, device=d)
    rc, sa = hop.hop_session_begin(mid, a_objs, 4, "sum", "f32", ce * 4, 2)
    assert rc == hop.HOP_OK
    rc, sb = hop.hop_session_begin(out, [b_objs[0], mid, b_objs[1]], 3, "sum", "f32", ce * 4, 2)
    assert rc == hop.HOP_OK
    assert hop.hop_session_ready(sb, 0, C) == hop.HOP_OK          # arrival order of the outer reduce: b0, mid, b1
    assert hop.hop_session_ready(sb, 1, 0) == hop.HOP_OK
    assert hop.hop_session_ready(sb, 2, C) == hop.HOP_OK
    seen = 0
    for c in range(1, C + 1):                                     # the inner participants stream chunk by chunk
        for i in range(4):
            assert hop.hop_session_ready(sa, i, c) == hop.HOP_OK
        done = hop.hop_session_chunks_final(sa)
        assert done == c
        if done > seen:
            assert hop.hop_session_ready(sb, 1, done) == hop.HOP_OK
            assert hop.hop_session_chunks_final(sb) == done       # the outer result follows chunk by chunk
            seen = done
    rca, info_a = hop.hop_session_finish(sa)
    rcb, info_b = hop.hop_session_finish(sb)
    torch.cuda.synchronize()
    assert rca == hop.HOP_OK and rcb == hop.HOP_OK and info_a["n_launches"] == C and info_b["n_launches"] == C
    _, inner, _, _ = oracle.reduce(a_vals, 4, oracle.SUM, oracle.F32, ce, 2, None, None)
    _, want, _, _ = oracle.reduce([b_vals[0], inner, b_vals[1]], 3, oracle.SUM, oracle.F32, ce, 2, None, None)
    assert np.array_equal(bits(workloads.to_numpy(mid)), bits(inner))
    assert np.array_equal(bits(workloads.to_numpy(out)), bits(want))


def test_adaptive_policy_changes_the_launches_not_the_bits():
    # eager, but partial progress only while the stream is idle: however the launches fall (it depends
    # on timing), the result is the oracle's, bit for bit; with failures and a late replacement
    d = dev()
    rng = np.random.default_rng(33)
    for dtype in ("f32", "bf16", "i32"):
        C, ce, n, k = 6, 8192, 9, 7
        E = C * ce - 5
        w = workloads.WORKLOADS[1].scaled(E * ES[dtype], ce * ES[dtype], n=n, k=k, dtype=dtype, tree_degree=3,
                                          dist={"f32": "uniform_pm1", "bf16": "normal_std1", "i32": "randint_pm2p20"}[dtype],
                                          order_seed=int(rng.integers(1 << 30)), data_seed=int(rng.integers(1 << 30)))
        objs = workloads.make_objects(w, device=d)
        order = w.ready_order()
        dst = torch.zeros_like(objs[0])
        rc, s = hop.hop_session_begin(dst, objs, k, "sum", dtype, w.chunk_bytes, 3)
        assert rc == hop.HOP_OK
        assert hop.hop_session_set_eager(s, 1) == hop.HOP_OK and hop.hop_session_set_adaptive(s, 1) == hop.HOP_OK
        failing = int(order[2])
        fm = np.full(n, -1, np.int64)
        fm[failing] = 2
        for c in range(1, C + 1):
            for i in order:
                i = int(i)
                if i == failing and c > 2:
                    continue
                assert hop.hop_session_ready(s, i, c) == hop.HOP_OK
                if c % 2 == 0:
                    torch.cuda.synchronize()                     # sometimes the stream is idle, sometimes not
            if c == 2:
                assert hop.hop_session_fail(s, failing) == hop.HOP_OK
        rc, info = hop.hop_session_finish(s)
        torch.cuda.synchronize()
        # the oracle on the final occupants: everybody announced itself at chunk 1, the failing one left after 2
        orc, want, k_eff, _ = oracle.reduce([workloads.to_numpy(o) for o in objs], k, oracle.SUM, ORA_DT[dtype], ce, 3,
                                            order, fm)
        assert rc == orc and info["k_eff"] == k_eff
        assert np.array_equal(bits(workloads.to_numpy(dst)), bits(want))


@pytest.mark.parametrize("dtype,mib", [("f32", 9), ("bf16", 17), ("i32", 33)])
def test_eager_segments_over_long_ranges(dtype, mib):
    # whole objects arrive one at a time and every arrival is folded into the saved accumulators at once: the
    # segment launches span the whole object, long enough for the layout with pieces 64 KiB apart (and, from
    # 20 MiB, the cap on resident waves). Same bits as the one-launch reduce and as the oracle on samples.
    d = dev()
    nbytes = mib * (1 << 20) + 5 * 1024 + 3 * 16 - ES[dtype]
    chunk = 3 << 20
    n, k, deg = 7, 6, 2
    w = workloads.Workload("eager_long_%s" % dtype, n=n, dtype=dtype, object_bytes=nbytes, chunk_bytes=chunk, k=k,
                           tree_degree=deg, ops=("sum",), order_seed=4242 + mib, data_seed=4343 + mib,
                           dist={"f32": "normal_std1", "bf16": "normal_std1", "i32": "randint_pm2p20"}[dtype])
    objs = workloads.make_objects(w, device=d)
    order = w.ready_order()
    fused = torch.zeros_like(objs[0])
    rc, info = hop.hop_reduce(fused, objs, k, "sum", dtype, chunk, deg, order, None)
    assert rc == hop.HOP_OK
    dst = torch.full_like(objs[0], 3)
    rc, s = hop.hop_session_begin(dst, objs, k, "sum", dtype, chunk, deg)
    assert rc == hop.HOP_OK and hop.hop_session_set_eager(s, 1) == hop.HOP_OK
    for i in order:
        assert hop.hop_session_ready(s, int(i), w.n_chunks) == hop.HOP_OK
    rc, sinfo = hop.hop_session_finish(s)
    torch.cuda.synchronize()
    assert rc == hop.HOP_OK and sinfo["n_launches"] >= k - 1
    assert torch.equal(dst.view(torch.int16 if dtype == "bf16" else torch.int32),
                       fused.view(torch.int16 if dtype == "bf16" else torch.int32))
    sampled_oracle_check(w, "sum", objs, [dst], rc, sinfo, np.random.default_rng(mib), per_chunk=16)


def test_readiness_by_event_needs_no_host_synchronisation():
    # The producers run on another stream: before each chunk of each object the producer stream is kept
    # busy with real work (passes over a 256 MiB buffer), then the chunk is written and an event recorded.
    # The session is told "ready after this event"; nobody waits on the host between producing and
    # reducing, and the session's stream has nothing else to wait for. Had it not waited for the events, it
    # would have read the zeros the objects held before. (A correct library can never fail this test,
    # however the host and the device are scheduled: only the result is checked, no timing.)
    d = dev()
    rng = np.random.default_rng(21)
    C, ce, n = 4, 4096, 5
    E = C * ce
    vals = [rng.standard_normal(E).astype(np.float32) for _ in range(n)]
    staged = [workloads.from_numpy(v, "f32", d) for v in vals]
    objs = [torch.zeros(E, device=d) for _ in range(n)]
    dst = torch.zeros(E, device=d)
    ballast = torch.zeros(64 << 20, device=d)
    producer, consumer = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    rc, s = hop.hop_session_begin(dst, objs, n, "sum", "f32", ce * 4, 2, stream=consumer.cuda_stream)
    assert rc == hop.HOP_OK
    order = [3, 0, 4, 1, 2]
    events = []
    for c in range(C):
        for i in order:
            with torch.cuda.stream(producer):
                for _ in range(4):
                    ballast.add_(1.0)                             # about half a millisecond of work in front of the data
                objs[i][c * ce:(c + 1) * ce].copy_(staged[i][c * ce:(c + 1) * ce])
                ev = torch.cuda.Event()
                ev.record(producer)
            events.append(ev)
            assert hop.hop_session_ready_after(s, i, c + 1, ev) == hop.HOP_OK
    rc, info = hop.hop_session_finish(s)
    assert rc == hop.HOP_OK and info["n_launches"] == C
    consumer.synchronize()                    # the consumer alone: if it had not waited for the producer, this returns early
    got = workloads.to_numpy(dst)
    torch.cuda.synchronize()
    _, want, _, _ = oracle.reduce(vals, n, oracle.SUM, oracle.F32, ce, 2, np.array(order, np.int32), None)
    assert np.array_equal(bits(got), bits(want))
    assert float(ballast[0]) == 4.0 * C * n


def test_other_stream():
    d = dev()
    w = workloads.WORKLOADS[1]
    objs = workloads.make_objects(w, device=d)
    dst = torch.zeros_like(objs[0])
    torch.cuda.synchronize()
    st = torch.cuda.Stream()
    rc, info = hop.hop_reduce(dst, objs, w.k, "sum", w.dtype, w.chunk_bytes, w.tree_degree, None, None, stream=st)
    st.synchronize()
    _, want, _, _ = oracle.reduce([workloads.to_numpy(o) for o in objs], w.k, oracle.SUM, oracle.F32,
                                  w.chunk_bytes // 4, w.tree_degree, None, None)
    assert rc == hop.HOP_OK and np.array_equal(bits(workloads.to_numpy(dst)), bits(want))


# ------------------------------------------------------------------ full-size workloads, sampled against the oracle

def sampled_oracle_check(w, op, objs, dsts, rc, info, rng, per_chunk=64):
    """The reduce is elementwise, so the oracle run on a gather of the same element positions from every
    object must equal the gather of the GPU result. Positions: first and last elements of every chunk
    plus random ones; per_chunk of them for each chunk so that the gathered objects keep the chunk count."""
    C, E = w.n_chunks, w.n_elems
    ce = w.chunk_bytes // ES[w.dtype]
    idx = []
    for c in range(C):
        lo, hi = c * ce, min((c + 1) * ce, E)
        pick = np.concatenate([[lo, lo + 1, hi - 2, hi - 1], rng.integers(lo, hi, size=per_chunk - 4)])
        idx.append(np.sort(pick))
    idx = torch.from_numpy(np.concatenate(idx)).to(dev())
    small = [workloads.to_numpy(o[idx]) for o in objs]
    d = info["degree_used"] if w.tree_degree == 0 else w.tree_degree
    orc, want, k_eff, n_rep = oracle.reduce(small, w.k, ORA_OP[op], ORA_DT[w.dtype], per_chunk, d, w.ready_order(),
                                            w.fail_mask())
    assert rc == orc and info["k_eff"] == k_eff and info["n_replaced"] == n_rep
    for dst in dsts:
        got = workloads.to_numpy(dst[idx])
        assert np.array_equal(bits(got), bits(want))
    return small, want


def full_oracle_check(w, op, objs, dsts, rc, info, order=None, fm=None):
    """Every element of the result against the oracle's tree-ordered reduce of the same inputs."""
    order = w.ready_order() if order is None else order
    d = info["degree_used"] if w.tree_degree == 0 else w.tree_degree
    host = [workloads.to_numpy(o) for o in objs]
    orc, want, k_eff, n_rep = oracle.reduce(host, w.k, ORA_OP[op], ORA_DT[w.dtype], max(1, w.chunk_bytes // ES[w.dtype]), d,
                                            order, fm)
    assert rc == orc and info["k_eff"] == k_eff and info["n_replaced"] == n_rep
    for dst in dsts:
        got = workloads.to_numpy(dst)
        assert np.array_equal(bits(got), bits(want)), "mismatch at %s" % np.flatnonzero(bits(got) != bits(want))[:8]
    return host, want


def free_order_check(w, host, got, order=None, fm=None, n_check=1 << 20):
    """A float sum against the order-free definition (the oracle's float64 sum over the occupants) within the
    tolerance for free ordering, on the first and last n_check elements."""
    order = w.ready_order() if order is None else order
    rc, occ, k_eff, _ = oracle.occupants(w.n, w.k, w.n_chunks, order, fm)
    assert rc >= 0
    tol = 1e-5 * np.log2(max(k_eff, 2)) if w.dtype == "f32" else 1e-2
    for part in (slice(0, n_check), slice(max(0, w.n_elems - n_check), w.n_elems)):
        small = [h[part] for h in host]
        ref = oracle.reduce_set(small, occ, oracle.SUM, ORA_DT[w.dtype])
        mag = np.zeros_like(ref)
        for o in occ:
            if o >= 0:
                x = small[o] if w.dtype == "f32" else oracle.bf16_to_f32(small[o])
                mag += np.abs(x.astype(np.float64))
        g = got[part] if w.dtype == "f32" else oracle.bf16_to_f32(got[part])
        assert np.all(np.abs(g.astype(np.float64) - ref) <= tol * np.maximum(np.abs(ref), mag / k_eff))


# every launch shape of the reduce kernel, each at a size just inside its range, with one object a few
# elements short of a tile so that the ragged end is exercised too: (dtype, n, k, degree, bytes short of or
# beyond a whole number of MiB, MiB, dist). From 3 MiB a workgroup's pieces lie 16 or 64 KiB apart, in
# groups of 32 or 256 KiB: "a few KiB beyond" leaves a last group in which most workgroups own nothing.
SHORT = -3 * 16                                    # not a whole tile, not a whole vector (minus one element below)
BEYOND = 5 * 1024 + 3 * 16                         # a last group with five whole pieces and a ragged sixth
LAUNCH_SHAPE_CASES = [
    ("f32", 6, 5, 2, SHORT, 2, "uniform_pm1"),       # 1 KiB tiles, 8 sources in flight (few tiles)
    ("f32", 6, 5, 2, SHORT, 6, "uniform_pm1"),       # 2 KiB tiles, 2 in flight, pieces 16 KiB apart
    ("f32", 6, 5, 2, BEYOND, 5, "uniform_pm1"),      # the same, a few KiB into the last group
    ("f32", 6, 5, 4, SHORT, 12, "normal_std1"),      # four pieces 64 KiB apart, uncapped
    ("f32", 6, 5, 4, BEYOND, 9, "normal_std1"),      # the same, a few KiB into the last group
    ("i32", 6, 6, 2, SHORT, 22, "randint_pm2p20"),   # four pieces 64 KiB apart, 8 waves per CU
    ("i32", 6, 6, 2, BEYOND, 21, "randint_pm2p20"),  # the same, a few KiB into the last group
    ("f32", 5, 4, 1, SHORT, 52, "normal_std1"),      # a chain over 52 MiB objects
    ("bf16", 6, 6, 6, SHORT, 50, "normal_std1"),     # bf16 at depth 1..2, four pieces
    ("bf16", 40, 40, 2, SHORT, 17, "normal_std1"),   # bf16 binary tree (5 levels): two pieces, two sources in flight
    ("bf16", 40, 40, 2, BEYOND, 5, "normal_std1"),   # the same below 8 MiB: pieces 16 KiB apart
    ("bf16", 12, 12, 4, SHORT, 20, "normal_std1"),   # bf16 at depth 2
    ("bf16", 16, 16, 2, BEYOND, 9, "normal_std1"),   # bf16 at depth 3..4: two pieces per workgroup, 64 KiB apart
    ("f32", 40, 40, 2, SHORT, 49, "normal_std1"),    # fp32 binary tree (5 levels)
]


@pytest.mark.parametrize("dtype,n,k,d,delta,mib,dist", LAUNCH_SHAPE_CASES)
def test_every_launch_shape_against_the_oracle(dtype, n, k, d, delta, mib, dist):
    nbytes = mib * (1 << 20) + delta - ES[dtype]
    chunk = 1 << 20
    w = workloads.Workload("shape_%s_%d" % (dtype, mib), n=n, dtype=dtype, object_bytes=nbytes, chunk_bytes=chunk,
                           k=k, tree_degree=d, ops=("sum",), dist=dist, order_seed=1234 + mib, data_seed=99 + mib)
    print("launch shape case", w.name, n, k, d, nbytes, flush=True)
    objs = workloads.make_objects(w, device=dev())
    dst = torch.zeros_like(objs[0])
    sel = [objs[i] for i in w.ready_order()[:k]]
    for op in ("sum", "max"):
        dst.fill_(7)                                  # a piece no workgroup wrote would keep this
        rc, info = hop.hop_reduce(dst, objs, k, op, dtype, chunk, d, w.ready_order(), None)
        torch.cuda.synchronize()
        assert rc == hop.HOP_OK and info["n_launches"] == 1
        rng = np.random.default_rng(mib)
        sampled_oracle_check(w, op, objs, [dst], rc, info, rng, per_chunk=16)
        # the very end of the object: the ragged vector and the elements before it
        tail = slice(w.n_elems - 40, w.n_elems)
        small = [workloads.to_numpy(o[tail]) for o in objs]
        _, want, _, _ = oracle.reduce(small, k, ORA_OP[op], ORA_DT[dtype], 40, d, w.ready_order(), None)
        assert np.array_equal(bits(workloads.to_numpy(dst[tail])), bits(want))
        if op == "sum":
            # every element against the oracle, and (floats) against the order-free definition within the
            # tolerance for free ordering
            host, want = full_oracle_check(w, op, objs, [dst], rc, info)
            if dtype != "i32":
                free_order_check(w, host, want)
        else:
            # max is exact in any order: every element against a plain running maximum
            ref = sel[0].clone()
            for o in sel[1:]:
                ref = torch.maximum(ref, o)
            assert torch.equal(dst, ref)


@pytest.mark.parametrize("dtype,mib,residues", [("f32", 2, (16,)), ("f32", 6, (16,)), ("f32", 12, (80,)), ("i32", 20, (112,)),
                                                ("bf16", 20, (16,)), ("f32", 9, (0, 16, 32, 48, 64, 80, 96, 112))])
def test_sources_that_are_only_16_byte_aligned(dtype, mib, residues):
    # objects carved from one buffer so that they start 16..112 bytes past a 128-byte boundary (all alike, or
    # every object differently), the result 48 bytes past one: the kernels start their grid of vectors at a
    # boundary of the sources and skip what lies in front of the range
    d = dev()
    n, k, deg = 6, 5, 2
    nbytes = mib * (1 << 20) + 5 * 1024 + 3 * 16 - ES[dtype]
    chunk = 1 << 20
    w = workloads.Workload("unaligned_%s_%d" % (dtype, mib), n=n, dtype=dtype, object_bytes=nbytes, chunk_bytes=chunk,
                           k=k, tree_degree=deg, ops=("sum",), order_seed=77 + mib, data_seed=88 + mib,
                           dist={"f32": "normal_std1", "bf16": "normal_std1", "i32": "randint_pm2p20"}[dtype])
    aligned = workloads.make_objects(w, device=d)
    E, es = w.n_elems, ES[dtype]
    slot = (nbytes + 1023) // 1024 * 1024 + 1024
    pool = torch.zeros((n + 1) * slot // es, dtype=aligned[0].dtype, device=d)
    assert pool.data_ptr() % 128 == 0
    objs = []
    for i, a in enumerate(aligned):
        at = (i * slot + residues[i % len(residues)]) // es
        pool[at:at + E].copy_(a)
        objs.append(pool[at:at + E])
        assert objs[-1].data_ptr() % 128 == residues[i % len(residues)]
    at = (n * slot + 48) // es
    dst = pool[at:at + E]
    sel = [objs[i] for i in w.ready_order()[:k]]
    for op in ("sum", "max"):
        dst.fill_(7)
        rc, info = hop.hop_reduce(dst, objs, k, op, dtype, chunk, deg, w.ready_order(), None)
        torch.cuda.synchronize()
        assert rc == hop.HOP_OK
        sampled_oracle_check(w, op, objs, [dst], rc, info, np.random.default_rng(mib), per_chunk=16)
        head = slice(0, 40)
        _, want, _, _ = oracle.reduce([workloads.to_numpy(o[head]) for o in objs], k, ORA_OP[op], ORA_DT[dtype], 40, deg,
                                      w.ready_order(), None)
        assert np.array_equal(bits(workloads.to_numpy(dst[head])), bits(want))
        if op == "sum":
            full_oracle_check(w, op, objs, [dst], rc, info)
        else:
            ref = sel[0].clone()
            for o in sel[1:]:
                ref = torch.maximum(ref, o)
            assert torch.equal(dst, ref)
    if mib in (9, 12):
        # the same objects through eager segments (every arrival folded into saved accumulators at once)
        rc, _ = hop.hop_reduce(dst, objs, k, "sum", dtype, chunk, deg, w.ready_order(), None)
        fused = dst.clone()
        dst.fill_(3)
        rc, ses = hop.hop_session_begin(dst, objs, k, "sum", dtype, chunk, deg)
        assert rc == hop.HOP_OK and hop.hop_session_set_eager(ses, 1) == hop.HOP_OK
        for i in w.ready_order():
            assert hop.hop_session_ready(ses, int(i), w.n_chunks) == hop.HOP_OK
        rc, _ = hop.hop_session_finish(ses)
        torch.cuda.synchronize()
        assert rc == hop.HOP_OK and torch.equal(dst.view(torch.int32), fused.view(torch.int32))
    # nothing outside the result was written: the bytes around it are still zero
    assert int(pool[at - 12:at].abs().sum()) == 0 and int(pool[at + E:at + E + 12].abs().sum()) == 0


def test_cfg2_full_size_every_element():
    w = workloads.WORKLOADS[2]
    print("full size", w.name, flush=True)
    objs = workloads.make_objects(w, device=dev())
    dst = torch.zeros_like(objs[0])
    rc, info = hop.hop_reduce(dst, objs, w.k, "sum", w.dtype, w.chunk_bytes, w.tree_degree, w.ready_order(), None)
    torch.cuda.synchronize()
    assert rc == hop.HOP_OK and info["n_launches"] == 1 and info["k_eff"] == 12
    host, want = full_oracle_check(w, "sum", objs, [dst], rc, info)
    # the order-free definition: the float64 sum over the first 12 ready, within the free-order tolerance
    free_order_check(w, host, want)


def test_cfg3_full_size_allreduce_every_element():
    w = workloads.WORKLOADS[3]
    print("full size", w.name, flush=True)
    objs = workloads.make_objects(w, device=dev())
    dsts = [torch.zeros_like(objs[0]) for _ in range(w.n_dst)]
    rc, info = hop.hop_allreduce(dsts, objs, w.k, "sum", w.dtype, w.chunk_bytes, w.tree_degree, w.ready_order(), None)
    torch.cuda.synchronize()
    assert rc == hop.HOP_OK and info["k_eff"] == 64
    # the first destination against the oracle, every element; the other 63 against the first
    host, want = full_oracle_check(w, "sum", objs, dsts[:1], rc, info)
    assert all(torch.equal(dsts[0], x) for x in dsts[1:])
    # integers are order-free: the oracle's unwrapped int64 sum over all 64, wrapped, is the same
    ref = oracle.reduce_set([h[:1 << 20] for h in host], np.arange(64, dtype=np.int32), oracle.SUM, oracle.I32)
    assert np.array_equal(ref.astype(np.int32), want[:1 << 20])


def test_cfg4_full_size_failure_every_element():
    w = workloads.WORKLOADS[4]
    print("full size", w.name, flush=True)
    objs = workloads.make_objects(w, device=dev())
    dst = torch.zeros_like(objs[0])
    rc, info = hop.hop_reduce(dst, objs, w.k, "sum", w.dtype, w.chunk_bytes, w.tree_degree, w.ready_order(),
                              w.fail_mask())
    torch.cuda.synchronize()
    # launch over chunks 0..9 that keeps the three subtree partials, their repair, chunks 10..31
    assert rc == hop.HOP_PARTIAL and info["k_eff"] == 31 and info["n_launches"] == 3
    assert info["chunks_redone"] == 10 * 5 and info["partial_stores"] == info["partial_loads"] == 10 * 3
    host, want = full_oracle_check(w, "sum", objs, [dst], rc, info, fm=w.fail_mask())
    # the order-free definition: within the bf16 tolerance of the float64 sum over the 31 survivors
    free_order_check(w, host, want, fm=w.fail_mask())
    del host
    # and independent of when the failure happened, and of whether partial results were kept
    dst2 = torch.zeros_like(dst)
    fm = w.fail_mask().copy()
    fm[7] = 31
    rc2, info2 = hop.hop_reduce(dst2, objs, w.k, "sum", w.dtype, w.chunk_bytes, w.tree_degree, w.ready_order(), fm)
    torch.cuda.synchronize()
    assert rc2 == hop.HOP_PARTIAL and info2["chunks_redone"] == 31 * 5
    assert torch.equal(dst.view(torch.int16), dst2.view(torch.int16))


# ------------------------------------------------------------------ failures repaired from kept partial results

KEPT_CASES = [
    # dtype, op, n, k, d, object bytes, chunk bytes, {object (by arrival rank): chunks before it fails}
    # (partial results are kept by launches over at least 8 MiB per object)
    ("bf16", "sum", 32, 32, 8, (32 << 20) + 6, 1 << 20, {28: 10}),             # workload 4's shape: a childless child of the root
    ("bf16", "sum", 32, 32, 8, (24 << 20) + 6, 1 << 20, {12: 9}),              # inside the second subtree
    ("f32", "sum", 16, 12, 2, (24 << 20) + 12, 2 << 20, {3: 5}),               # binary tree, replaced by a waiting object
    ("f32", "max", 40, 40, 4, (20 << 20) + 4, 1 << 20, {0: 9, 30: 17}),         # two failures at different times
    ("i32", "sum", 64, 60, 16, 16 << 20, 512 << 10, {5: 24, 59: 24, 61: 3}),    # two at once, and a waiting object that dies too
    ("bf16", "min", 24, 24, 3, (20 << 20) + 2, 4 << 20, {23: 2}),               # the last arrival; three levels of accumulators
    ("f32", "sum", 12, 12, 4, 24 << 20, 8 << 20, {5: 1}),                       # the root itself
    ("f32", "sum", 32, 32, 2, (16 << 20) + 8, 4 << 20, {19: 2}),                # deep binary tree: subtrees two levels down are kept
    ("i32", "max", 48, 48, 2, 24 << 20, 4 << 20, {2: 2, 40: 4}),                # the first repair keeps its subtree again, the second reads all four
]


@pytest.mark.parametrize("dtype,op,n,k,d,nbytes,chunk,fails", KEPT_CASES)
def test_failure_repaired_from_kept_partials_equals_oracle(dtype, op, n, k, d, nbytes, chunk, fails):
    base = workloads.WORKLOADS[{"f32": 2, "bf16": 4, "i32": 3}[dtype]]
    w = base.scaled(nbytes, chunk, n=n, k=k, tree_degree=d, order_seed=77 + n, data_seed=88 + k, fail={}, n_dst=0,
                    name="kept_%s_%d" % (dtype, n))
    order = w.ready_order()
    fm = np.full(n, -1, np.int64)
    for rank, c in fails.items():
        fm[order[rank]] = c
    rc, info = run_both(w, op, order=order, fm=fm)
    # partial results were kept by the launches made while participants could still fail, and read by the repairs
    assert info["partial_stores"] > 0 and info["partial_loads"] > 0, info
    # the same call without keeping gives the same bits with more re-reading (checked against the oracle
    # by run_both above; here: through a session with retention switched off)
    objs = workloads.make_objects(w, device=dev())
    dst_a, dst_b = torch.zeros_like(objs[0]), torch.zeros_like(objs[0])
    infos = []
    for dst, keep in ((dst_a, True), (dst_b, False)):
        src, s = hop.hop_session_begin(dst, objs, k, op, dtype, chunk, d)
        assert src == hop.HOP_OK and hop.hop_session_set_retention(s, keep) == hop.HOP_OK
        alive = [int(i) for i in order if fm[i] != 0]
        for i in alive:
            assert hop.hop_session_ready(s, i, 0) == hop.HOP_OK
        C = w.n_chunks
        for step in sorted({int(c) for c in fm if 0 < c < C}) + [C]:
            for i in list(alive):
                lim = C if fm[i] < 0 or fm[i] >= C else int(fm[i])
                assert hop.hop_session_ready(s, i, min(step, lim)) == hop.HOP_OK
            for i in list(alive):
                if 0 < fm[i] < C and fm[i] == step:
                    assert hop.hop_session_fail(s, i) == hop.HOP_OK
                    alive.remove(i)
        src, inf = hop.hop_session_finish(s)
        assert src == rc
        infos.append(inf)
    torch.cuda.synchronize()
    assert torch.equal(dst_a.view(torch.int16), dst_b.view(torch.int16))
    assert infos[1]["partial_stores"] == 0 and infos[0]["partial_loads"] > 0
    assert infos[0]["chunk_steps"] < infos[1]["chunk_steps"]


def test_allreduce_with_a_failure_keeps_partials_and_all_destinations_agree():
    w = workloads.WORKLOADS[3].scaled(16 << 20, 1 << 20, n=20, k=20, tree_degree=4, n_dst=5, name="kept_allreduce")
    objs = workloads.make_objects(w, device=dev())
    order = w.ready_order()
    fm = np.full(w.n, -1, np.int64)
    fm[order[9]] = 9
    dsts = [torch.full_like(objs[0], -5) for _ in range(w.n_dst)]
    rc, info = hop.hop_allreduce(dsts, objs, w.k, "sum", w.dtype, w.chunk_bytes, w.tree_degree, order, fm)
    torch.cuda.synchronize()
    assert rc == hop.HOP_PARTIAL and info["k_eff"] == 19 and info["partial_loads"] > 0
    orc, outs, _, _ = oracle.allreduce([workloads.to_numpy(o) for o in objs], w.n_dst, w.k, oracle.SUM, oracle.I32,
                                       w.chunk_bytes // 4, w.tree_degree, order, fm)
    assert orc == rc
    for got, want in zip(dsts, outs):
        assert np.array_equal(workloads.to_numpy(got), want)


def test_late_arrival_into_a_hole_reuses_the_kept_partials():
    # 9 objects, binary tree on 8 positions; chunk by chunk; the 6th arrival fails after 3 chunks with nobody
    # waiting (a hole), later a 9th object arrives and takes the hole: the chunks produced in between are
    # repaired twice, each time from the partials of the subtree that did not change
    w = workloads.WORKLOADS[2].scaled(64 << 20, 8 << 20, n=9, k=8, tree_degree=2, order_seed=None, name="kept_late")
    objs = workloads.make_objects(w, device=dev())
    dst = torch.zeros_like(objs[0])
    C = w.n_chunks
    rc, s = hop.hop_session_begin(dst, objs, w.k, "sum", w.dtype, w.chunk_bytes, w.tree_degree)
    assert rc == hop.HOP_OK
    for i in range(8):
        assert hop.hop_session_ready(s, i, 0) == hop.HOP_OK
    for c in range(1, 4):
        for i in range(8):
            assert hop.hop_session_ready(s, i, c) == hop.HOP_OK
    assert hop.hop_session_chunks_final(s) == 3
    assert hop.hop_session_fail(s, 5) == hop.HOP_OK
    for c in range(4, 6):
        for i in range(8):
            if i != 5:
                assert hop.hop_session_ready(s, i, c) == hop.HOP_OK
    assert hop.hop_session_chunks_final(s) == 5
    assert hop.hop_session_ready(s, 8, C) == hop.HOP_OK          # the late arrival, complete
    for i in range(8):
        if i != 5:
            assert hop.hop_session_ready(s, i, C) == hop.HOP_OK
    rc, info = hop.hop_session_finish(s)
    torch.cuda.synchronize()
    assert rc == hop.HOP_OK and info["k_eff"] == 8 and info["n_replaced"] == 1 and info["partial_loads"] > 0
    order = np.array([0, 1, 2, 3, 4, 8, 6, 7, 5], np.int32)       # final placement: 8 sits where 5 was
    fm = np.full(9, -1, np.int64)
    fm[5] = 0
    orc, want, _, _ = oracle.reduce([workloads.to_numpy(o) for o in objs], 8, oracle.SUM, oracle.F32, w.chunk_bytes // 4, 2,
                                    order, fm)
    assert orc == hop.HOP_OK and np.array_equal(bits(workloads.to_numpy(dst)), bits(want))


def test_session_with_a_workspace_of_the_callers():
    # every byte of scratch (staged segments, saved accumulators, kept partials) from a buffer of the
    # caller's: same bits as the oracle and as a session on the library's own caches
    d = dev()
    w = workloads.WORKLOADS[2].scaled((12 << 20) + 12, 1 << 20, n=14, k=12, tree_degree=3, order_seed=31, data_seed=32,
                                      fail={}, name="own_workspace")
    objs = workloads.make_objects(w, device=d)
    order = w.ready_order()
    fm = np.full(w.n, -1, np.int64)
    fm[order[4]] = 9
    C = w.n_chunks
    need = hop.hop_workspace_bytes(w.n, w.k, w.object_bytes, w.chunk_bytes, w.tree_degree, w.dtype,
                                   policy=hop.HOP_WS_EAGER | hop.HOP_WS_FAILURES)
    assert need > 3 * w.n_elems * 4
    host = [workloads.to_numpy(o) for o in objs]
    orc, want, k_eff, _ = oracle.reduce(host, w.k, oracle.SUM, oracle.F32, w.chunk_bytes // 4, w.tree_degree, order, fm)
    for eager in (0, 1):
        ws = torch.empty(need + (1 << 20), dtype=torch.uint8, device=d)        # + room for the staged segments
        dst = torch.zeros_like(objs[0])
        rc, info = session_replay(objs, dst, w.k, "sum", w.dtype, w.chunk_bytes, w.tree_degree, order, fm, C, fine=False,
                                  eager=eager, workspace=ws)
        torch.cuda.synchronize()
        assert rc == orc and info["k_eff"] == k_eff
        assert np.array_equal(bits(workloads.to_numpy(dst)), bits(want))
        if eager == 0:
            assert info["partial_stores"] > 0 and info["partial_loads"] > 0       # kept partials lived in the workspace
    # many small objects: the table of the one-launch form of the program comes out of the workspace too, one
    # per version of the program (each failure makes a new one); hop_workspace_bytes counts one
    wm = workloads.WORKLOADS[5].scaled(3000 * 4, 4096, n=400, k=380, tree_degree=8, order_seed=33, data_seed=34,
                                       fail={}, name="own_workspace_small", n_dst=0)
    mobjs = workloads.make_objects(wm, device=d)
    morder = wm.ready_order()
    mfm = np.full(wm.n, -1, np.int64)
    mfm[morder[7]], mfm[morder[200]] = 1, 2
    per_version = hop.hop_workspace_bytes(wm.n, wm.k, wm.object_bytes, wm.chunk_bytes, wm.tree_degree, wm.dtype)
    assert per_version >= 380 // 8 * 192
    ws = torch.empty(4 * per_version, dtype=torch.uint8, device=d)
    mdst = torch.zeros_like(mobjs[0])
    rc, info = session_replay(mobjs, mdst, wm.k, "sum", wm.dtype, wm.chunk_bytes, wm.tree_degree, morder, mfm, wm.n_chunks,
                              fine=True, workspace=ws)
    torch.cuda.synchronize()
    morc, mwant, mk_eff, _ = oracle.reduce([workloads.to_numpy(o) for o in mobjs], wm.k, oracle.SUM, oracle.F32,
                                           wm.chunk_bytes // 4, wm.tree_degree, morder, mfm)
    assert rc == morc and info["k_eff"] == mk_eff
    assert np.array_equal(bits(workloads.to_numpy(mdst)), bits(mwant))
    # two thousand bf16 objects of 100 KiB (more values alive at a time than the one-launch form has room for): the
    # program is cut into sub-programs whose partial results (4-byte accumulators in whole blocks) and records
    # come out of the workspace, which the library sized itself
    wb = workloads.WORKLOADS[4].scaled(100 * 1024 + 6, 16 * 2100, n=2000, k=1990, tree_degree=16, order_seed=35, data_seed=36,
                                       fail={}, name="own_workspace_cut", n_dst=0)
    assert not takes_the_one_launch_path(wb, wide=True)
    bobjs = workloads.make_objects(wb, device=d)
    border = wb.ready_order()
    need_cut = hop.hop_workspace_bytes(wb.n, wb.k, wb.object_bytes, wb.chunk_bytes, wb.tree_degree, wb.dtype)
    assert need_cut >= 50 * 2 * 16 * 2100                 # dozens of subtrees, twice the bytes of a chunk each
    ws = torch.zeros(need_cut, dtype=torch.uint8, device=d)
    bdst = torch.zeros_like(bobjs[0])
    rc, info = session_replay(bobjs, bdst, wb.k, "sum", wb.dtype, wb.chunk_bytes, wb.tree_degree, border, None, wb.n_chunks,
                              fine=False, workspace=ws)
    torch.cuda.synchronize()
    borc, bwant, bk_eff, _ = oracle.reduce([workloads.to_numpy(o) for o in bobjs], wb.k, oracle.SUM, oracle.BF16,
                                           wb.chunk_bytes // 2, wb.tree_degree, border, None)
    assert rc == borc and info["k_eff"] == bk_eff
    assert np.array_equal(bits(workloads.to_numpy(bdst)), bits(bwant))
    # the cut was made (a workspace too small for it would have sent the call down the plain path, which leaves
    # only the staged program behind): the partial results are still there
    assert int((ws != 0).sum()) > 50 * wb.object_bytes
    # a workspace that cannot hold the saved accumulators: the event that needs them says so
    small = torch.empty(1 << 20, dtype=torch.uint8, device=d)
    dst = torch.zeros_like(objs[0])
    rc, s = hop.hop_session_begin(dst, objs, w.k, "sum", w.dtype, w.chunk_bytes, w.tree_degree)
    assert rc == hop.HOP_OK and hop.hop_session_set_workspace(s, small) == hop.HOP_OK
    assert hop.hop_session_set_eager(s, 1) == hop.HOP_OK
    assert hop.hop_session_ready(s, int(order[0]), C) == hop.HOP_ERR_TOO_LARGE
    hop.hop_session_finish(s)
    # too late once something has been staged; misaligned memory is refused
    rc, s = hop.hop_session_begin(dst, objs, w.k, "sum", w.dtype, w.chunk_bytes, w.tree_degree)
    assert hop.hop_session_set_eager(s, 1) == hop.HOP_OK
    assert hop.hop_session_ready(s, int(order[0]), C) == hop.HOP_OK
    assert hop.hop_session_set_workspace(s, small) == hop.HOP_ERR_INVALID
    assert hop.hop_session_set_workspace(s, int(small.data_ptr()) + 16, 1 << 19) == hop.HOP_ERR_ALIGN
    hop.hop_session_finish(s)
    torch.cuda.synchronize()


def test_eager_session_with_a_workspace_can_be_captured_in_a_graph():
    # with a workspace of the caller's an eager session is nothing but kernel launches: its event calls can
    # be recorded into a graph, and every replay must see the current inputs
    d = dev()
    w = workloads.WORKLOADS[2].scaled((2 << 20) + 12, 512 << 10, n=6, k=6, tree_degree=2, order_seed=41, data_seed=42,
                                      name="captured_session")
    objs = workloads.make_objects(w, device=d)
    order = w.ready_order()
    dst = torch.zeros_like(objs[0])
    need = hop.hop_workspace_bytes(w.n, w.k, w.object_bytes, w.chunk_bytes, w.tree_degree, w.dtype, policy=hop.HOP_WS_EAGER)
    ws = torch.empty(need + (256 << 10), dtype=torch.uint8, device=d)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        rc, info = session_replay(objs, dst, w.k, "sum", w.dtype, w.chunk_bytes, w.tree_degree, order, None, w.n_chunks,
                                  fine=False, eager=1, workspace=ws)
    assert rc == hop.HOP_OK and info["n_launches"] == w.k
    rng = np.random.default_rng(6)
    for rep in range(3):
        for o in objs:                                # eager work between the replays
            o.mul_(float(rng.uniform(0.5, 1.5)))
        dst.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        _, want, _, _ = oracle.reduce([workloads.to_numpy(o) for o in objs], w.k, oracle.SUM, oracle.F32,
                                      w.chunk_bytes // 4, w.tree_degree, order, None)
        assert np.array_equal(bits(workloads.to_numpy(dst)), bits(want)), rep


def test_calibration_feeds_the_automatic_degree():
    rc, lat, bw = hop.hop_calibrate()
    assert rc == hop.HOP_OK
    # a dependent launch costs microseconds, the reduce streams at terabytes per second (MI355X peak: 8)
    assert 2e-7 < lat < 1e-4 and 1e12 < bw < 8e12, (lat, bw)
    for k, nbytes in ((64, 16 << 20), (12, 64 << 20), (1000, 4096), (5, 1 << 20)):
        assert hop.hop_pick_degree(k, nbytes) == hop.hop_pick_degree(k, nbytes, lat, bw)
    # tree_degree 0 uses it, and the result is the oracle's for the degree reported
    w = workloads.WORKLOADS[3].scaled(256 << 10, 16 << 10, n_dst=0)
    rc, info = run_both(w, "sum")
    assert rc == hop.HOP_OK and info["degree_used"] == hop.hop_pick_degree(w.k, w.object_bytes, lat, bw)


def test_repeated_small_calls_replay_their_recorded_launches_correctly():
    # a failure-free call over small inputs is recorded the first time and replayed afterwards; every
    # replay must land in the destination of that call and see the objects' current contents, and
    # anything that changes the schedule (order, k, degree, another object) must not hit the recording
    d = dev()
    w = workloads.WORKLOADS[5]
    objs = workloads.make_objects(w, device=d)
    order = w.ready_order()

    def check(objs_now, order_now, k, deg, stream=None):
        dst = torch.full_like(objs_now[0], -3)
        rc, info = hop.hop_reduce(dst, objs_now, k, "sum", w.dtype, w.chunk_bytes, deg, order_now, None, stream=stream)
        if stream is not None:
            stream.synchronize()
        torch.cuda.synchronize()
        orc, want, k_eff, _ = oracle.reduce([workloads.to_numpy(o) for o in objs_now], k, oracle.SUM, oracle.F32,
                                            w.chunk_bytes // 4, deg, order_now, None)
        assert rc == orc == hop.HOP_OK and info["k_eff"] == k_eff
        assert np.array_equal(bits(workloads.to_numpy(dst)), bits(want))
        return info
    first = check(objs, order, w.k, w.tree_degree)
    for rep in range(3):                               # replays: new destination each time, contents changed in place
        objs[int(order[rep])].mul_(1.5)
        assert check(objs, order, w.k, w.tree_degree) == first
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    check(objs, order, w.k, w.tree_degree, stream=st)            # another stream shares the recording's scratch
    check(objs, order, w.k, w.tree_degree)
    order2 = order.copy()
    order2[[0, 1]] = order2[[1, 0]]
    check(objs, order2, w.k, w.tree_degree)                      # another arrival order: another schedule
    check(objs, order, w.k - 1, w.tree_degree)
    check(objs, order, w.k, 4)
    swapped = list(objs)
    swapped[3], swapped[4] = swapped[4], swapped[3]
    check(swapped, order, w.k, w.tree_degree)
    # more distinct calls than recordings are kept: the oldest ones make room and are simply planned again
    for i in range(140):
        check(objs[:200 + i], np.arange(200 + i, dtype=np.int32), 150 + i, 8)
    check(objs, order, w.k, w.tree_degree)
    assert hop.hop_shutdown() == hop.HOP_OK                      # frees the recordings too
    check(objs, order, w.k, w.tree_degree)
    check(objs, order, w.k, w.tree_degree)


def test_recordings_that_hold_much_scratch_make_room_for_each_other():
    # calls over thousands of medium objects are recorded with the partial results of their sub-programs (tens
    # of MiB each); together the recordings may hold 1 GiB, then the least recently used ones go. 90 distinct
    # calls (k differs) of about 15 MiB each pass that limit; every result, recorded, replayed or planned again
    # after its recording went, equals the oracle's
    d = dev()
    w = workloads.WORKLOADS[5].scaled(128 << 10, 128 << 10, n=2000, k=2000, tree_degree=16, order_seed=21, data_seed=22,
                                      fail={}, name="big_recordings", n_dst=0)
    objs = workloads.make_objects(w, device=d)
    host = [workloads.to_numpy(o) for o in objs]
    order = w.ready_order()

    def check(k, with_oracle):
        dst = torch.full_like(objs[0], -1)
        rc, info = hop.hop_reduce(dst, objs, k, "sum", w.dtype, w.chunk_bytes, w.tree_degree, order, None)
        torch.cuda.synchronize()
        assert rc == hop.HOP_OK and info["k_eff"] == k
        if with_oracle:
            _, want, _, _ = oracle.reduce(host, k, oracle.SUM, oracle.F32, w.chunk_bytes // 4, w.tree_degree, order, None)
            assert np.array_equal(bits(workloads.to_numpy(dst)), bits(want)), k
        return workloads.to_numpy(dst)
    first = {}
    for k in range(1900, 1990):
        first[k] = check(k, k % 15 == 0)
    for k in (1900, 1945, 1989, 1901):                  # gone and planned again, or still recorded: the same bits
        assert np.array_equal(bits(check(k, False)), bits(first[k]))
    assert hop.hop_shutdown() == hop.HOP_OK


def test_a_known_shape_over_other_buffers_fills_in_the_addresses_only():
    # a serving loop that gets fresh buffers for every request: the call's shape (order, k, degree, sizes) is
    # known from an earlier call, only the addresses are new; the one-launch form is reused with them. Every
    # call must read ITS objects (none of an earlier set), whatever mixture of known and new shapes comes by.
    d = dev()
    w = workloads.WORKLOADS[5]
    order = w.ready_order()
    rng = np.random.default_rng(77)

    def fresh_set(n):
        return [torch.from_numpy(rng.standard_normal(w.object_bytes // 4).astype(np.float32)).to(d) for _ in range(n)]

    def check(objs_now, order_now, k, deg, op="sum"):
        dst = torch.full_like(objs_now[0], -3)
        rc, info = hop.hop_reduce(dst, objs_now, k, op, w.dtype, w.chunk_bytes, deg, order_now, None)
        torch.cuda.synchronize()
        orc, want, k_eff, _ = oracle.reduce([workloads.to_numpy(o) for o in objs_now], k, ORA_OP[op], oracle.F32,
                                            w.chunk_bytes // 4, deg, order_now, None)
        assert rc == orc == hop.HOP_OK and info["k_eff"] == k_eff and info["n_launches"] == 1
        assert np.array_equal(bits(workloads.to_numpy(dst)), bits(want))
        return info
    sets = [fresh_set(w.n) for _ in range(4)]
    first = check(sets[0], order, w.k, w.tree_degree)
    for objs in sets[1:] + sets[:2]:                   # new addresses, then addresses seen before (recorded calls)
        assert check(objs, order, w.k, w.tree_degree) == first
    # what changes the schedule is another shape: other order, k, degree, op, number of objects
    order2 = order.copy()
    order2[[5, 9]] = order2[[9, 5]]
    check(sets[2], order2, w.k, w.tree_degree)
    check(sets[3], order2, w.k, w.tree_degree)
    check(sets[1], order, w.k - 3, w.tree_degree)
    check(sets[2], order, w.k, 5)
    check(sets[3], order, w.k, w.tree_degree, op="max")
    check(sets[0][:300], np.arange(300, dtype=np.int32), 280, 16)
    check(sets[1][:300], None, 280, 16)                # the identity order given as no order: another key, same result
    check(sets[2][:300], None, 280, 16)
    # more shapes than are kept
    for i in range(40):
        check(sets[i % 4][:100 + i], None, 90 + i, 8)
        check(sets[(i + 1) % 4][:100 + i], None, 90 + i, 8)
    assert check(sets[3], order, w.k, w.tree_degree) == first
    # all-reduces of one shape over fresh buffers: the reduce from the known form, then the copy
    for objs in sets:
        dsts = [torch.full_like(objs[0], 9) for _ in range(3)]
        rc, info = hop.hop_allreduce(dsts, objs, w.k, "sum", w.dtype, w.chunk_bytes, w.tree_degree, order, None)
        torch.cuda.synchronize()
        orc, outs, _, _ = oracle.allreduce([workloads.to_numpy(o) for o in objs], 3, w.k, oracle.SUM, oracle.F32,
                                           w.chunk_bytes // 4, w.tree_degree, order, None)
        assert rc == orc == hop.HOP_OK and info["n_launches"] == 1
        for got, want in zip(dsts, outs):
            assert np.array_equal(bits(workloads.to_numpy(got)), bits(want))
    assert hop.hop_shutdown() == hop.HOP_OK
    assert check(sets[2], order, w.k, w.tree_degree) == first
    assert check(sets[1], order, w.k, w.tree_degree) == first
    # the same with objects of 96 KiB, whose shape is remembered in the wide one-launch form
    w = workloads.WORKLOADS[5].scaled(96 * 1024, 96 * 1024, n=150, k=140, tree_degree=8, order_seed=7, data_seed=8, fail={},
                                      name="known_wide", n_dst=0)
    assert takes_the_one_launch_path(w, wide=True)
    order = w.ready_order()
    sets = [fresh_set(w.n) for _ in range(3)]
    first = check(sets[0], order, w.k, w.tree_degree)
    for objs in sets[1:] + sets[:2]:
        assert check(objs, order, w.k, w.tree_degree) == first


def test_two_host_threads_on_their_own_streams_and_shutdown():
    import threading
    d = dev()
    w = workloads.WORKLOADS[2].scaled(1 << 20, 64 << 10)
    objs = workloads.make_objects(w, device=d)
    host = [workloads.to_numpy(o) for o in objs]
    order = w.ready_order()
    _, want, _, _ = oracle.reduce(host, w.k, oracle.SUM, oracle.F32, w.chunk_bytes // 4, w.tree_degree, order, None)
    torch.cuda.synchronize()
    errors = []

    def worker(seed):
        try:
            st = torch.cuda.Stream()
            dst = torch.zeros_like(objs[0])
            for _ in range(50):
                rc, info = hop.hop_reduce(dst, objs, w.k, "sum", w.dtype, w.chunk_bytes, w.tree_degree, order, None,
                                          stream=st)
                assert rc == hop.HOP_OK
            st.synchronize()
            assert np.array_equal(bits(workloads.to_numpy(dst)), bits(want))
        except Exception as e:            # noqa: BLE001 - reported to the main thread
            errors.append(repr(e))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(4)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    torch.cuda.synchronize()
    # the same with many small objects: every thread brings buffers of its own for one shape, so recordings and
    # the shape's one-launch form are looked up, inserted and evicted from four threads at once
    ws = workloads.WORKLOADS[5].scaled(2048, 2048, n=300, k=280, tree_degree=8, order_seed=9, data_seed=10, fail={},
                                       name="threads_small", n_dst=0)
    sorder = ws.ready_order()

    def small_worker(seed):
        try:
            rng = np.random.default_rng(seed)
            st = torch.cuda.Stream()
            for rep in range(40):
                vals = [rng.standard_normal(ws.object_bytes // 4).astype(np.float32) for _ in range(ws.n)]
                sobjs = [torch.from_numpy(v).to(d) for v in vals]
                sdst = torch.zeros_like(sobjs[0])
                st.wait_stream(torch.cuda.current_stream())
                rc, info = hop.hop_reduce(sdst, sobjs, ws.k, "sum", ws.dtype, ws.chunk_bytes, ws.tree_degree, sorder, None,
                                          stream=st)
                st.synchronize()
                _, swant, _, _ = oracle.reduce(vals, ws.k, oracle.SUM, oracle.F32, ws.chunk_bytes // 4, ws.tree_degree,
                                               sorder, None)
                assert rc == hop.HOP_OK and np.array_equal(bits(workloads.to_numpy(sdst)), bits(swant)), rep
        except Exception as e:            # noqa: BLE001 - reported to the main thread
            errors.append(repr(e))

    threads = [threading.Thread(target=small_worker, args=(100 + i,)) for i in range(4)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    torch.cuda.synchronize()
    assert hop.hop_shutdown() == hop.HOP_OK          # cached workspaces freed; the library keeps working after
    dst = torch.zeros_like(objs[0])
    rc, _ = hop.hop_reduce(dst, objs, w.k, "sum", w.dtype, w.chunk_bytes, w.tree_degree, order, None)
    torch.cuda.synchronize()
    assert rc == hop.HOP_OK and np.array_equal(bits(workloads.to_numpy(dst)), bits(want))


def test_objects_larger_than_4_gib_use_64_bit_offsets():
    d = dev()
    n_elems = (1 << 30) + 1024 + 3                  # 4 GiB + 4 KiB + 12 bytes of int32: tail included
    a = torch.arange(n_elems, dtype=torch.int32, device=d)
    b = torch.full((n_elems,), 7, dtype=torch.int32, device=d)
    b[-5:] = torch.tensor([1, 2, 3, 4, 5], dtype=torch.int32, device=d)
    dst = torch.zeros(n_elems, dtype=torch.int32, device=d)
    print("large object", n_elems * 4, flush=True)
    rc, info = hop.hop_reduce(dst, [a, b], 2, "sum", "i32", 256 << 20, 1, None, None)
    torch.cuda.synchronize()
    assert rc == hop.HOP_OK and info["n_launches"] == 1
    assert torch.equal(dst, a + b)
    # and a failure beyond the 4 GiB mark: chunks 0..16 (of 17) are produced twice
    c = torch.ones(n_elems, dtype=torch.int32, device=d)
    rc, info = hop.hop_reduce(dst, [a, b, c], 2, "max", "i32", 256 << 20, 2, None, [-1, 16, -1])
    torch.cuda.synchronize()
    assert rc == hop.HOP_OK and info["n_replaced"] == 1 and info["chunks_redone"] == 16 * 2
    assert torch.equal(dst, torch.maximum(a, c))


def test_a_captured_call_that_would_need_cached_memory_is_refused():
    # programs of more than 128 steps and long chain tables are staged in blocks that go back to the library's
    # cache when the call ends: a graph cannot own them, so under capture such a call fails loudly instead of
    # leaving a graph whose replays read rewritten memory. hop_reduce_noalloc is the call for that (tested with
    # its own).
    d = dev()
    for nbytes, n in ((512, 6000), (2 << 20, 200)):         # more chains than ride in the kernel arguments; a staged program
        w = workloads.WORKLOADS[5].scaled(nbytes, nbytes, n=n, k=n, tree_degree=16, order_seed=3, data_seed=4, fail={},
                                          name="captured", n_dst=0)
        objs = workloads.make_objects(w, device=d)
        dst = torch.zeros_like(objs[0])
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            dst.zero_()
            rc, _ = hop.hop_reduce(dst, objs, w.k, "sum", w.dtype, w.chunk_bytes, w.tree_degree, None, None)
        assert rc == hop.HOP_ERR_CAPTURE and "captured" in hop.hop_strerror(rc)
        # outside the capture the same call works
        rc, _ = run_both(w, "sum", objs=objs)
        assert rc == hop.HOP_OK


def test_a_call_over_many_small_objects_can_be_captured_when_its_table_rides_in_the_arguments():
    # up to 256 chains travel inside the kernel arguments, which a graph node keeps: workload 5 through plain
    # hop_reduce, recorded and replayed with other contents in the same buffers
    d = dev()
    w = workloads.WORKLOADS[5]
    objs = workloads.make_objects(w, device=d)
    order = w.ready_order()
    dst = torch.zeros_like(objs[0])
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        rc, info = hop.hop_reduce(dst, objs, w.k, "sum", w.dtype, w.chunk_bytes, w.tree_degree, order, None)
    assert rc == hop.HOP_OK and info["n_launches"] == 1
    rng = np.random.default_rng(19)
    for rep in range(3):
        for o in objs[::41]:
            o.mul_(float(rng.uniform(0.5, 1.5)))
        dst.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        _, want, _, _ = oracle.reduce([workloads.to_numpy(o) for o in objs], w.k, oracle.SUM, oracle.F32,
                                      w.chunk_bytes // 4, w.tree_degree, order, None)
        assert np.array_equal(bits(workloads.to_numpy(dst)), bits(want)), rep


@pytest.mark.parametrize("object_mib", [1, 49])
def test_reduce_can_be_captured_in_a_graph_and_replayed(object_mib):
    # short programs ride in the kernel arguments: a call is nothing but kernel launches on the
    # caller's stream, so it can be recorded into a graph; every replay must see the current inputs.
    # 49 MiB objects take the launch shape that caps resident waves with a dynamic LDS allocation.
    d = dev()
    w = workloads.WORKLOADS[1].scaled(object_mib << 20)
    objs = workloads.make_objects(w, device=d)
    dst = torch.zeros_like(objs[0])
    order = w.ready_order()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        rc, info = hop.hop_reduce(dst, objs, w.k, "sum", w.dtype, w.chunk_bytes, w.tree_degree, order, None)
    assert rc == hop.HOP_OK
    rng = np.random.default_rng(5)
    for rep in range(3):
        for o in objs:                                # eager work between the replays
            o.mul_(float(rng.uniform(0.5, 1.5)))
        dst.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        _, want, _, _ = oracle.reduce([workloads.to_numpy(o) for o in objs], w.k, oracle.SUM, oracle.F32,
                                      w.chunk_bytes // 4, w.tree_degree, order, None)
        assert np.array_equal(bits(workloads.to_numpy(dst)), bits(want)), rep
