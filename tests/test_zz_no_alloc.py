"""GPU test of hop_reduce_noalloc, the entry point that allocates nothing on the device: its output
must equal hop_reduce's (and the oracle's) bit for bit, also when a call follows a larger one whose
partial results and programs are still lying in the shared static scratch."""
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


def bits(a):
    return a.view(np.uint32) if a.dtype == np.float32 else a


def both_entry_points(w, op, fm=None):
    """The workload through hop_reduce_noalloc and through hop_reduce; both against the oracle."""
    dev = torch.device("cuda:0")
    objs = workloads.make_objects(w, device=dev)
    order = w.ready_order()
    print("case", w.name, w.dtype, op, "n", w.n, "k", w.k, "bytes", w.object_bytes, "d", w.tree_degree, flush=True)
    dst_static = torch.full_like(objs[0], 55)
    dst_plain = torch.full_like(objs[0], 66)
    rc_s, info_s = hop.hop_reduce_noalloc(dst_static, objs, w.k, op, w.dtype, w.chunk_bytes, w.tree_degree, order, fm)
    rc_p, info_p = hop.hop_reduce(dst_plain, objs, w.k, op, w.dtype, w.chunk_bytes, w.tree_degree, order, fm)
    torch.cuda.synchronize()
    assert rc_s == rc_p and rc_s >= 0, (rc_s, rc_p)
    assert info_s["degree_used"] == info_p["degree_used"]
    got_s, got_p = workloads.to_numpy(dst_static), workloads.to_numpy(dst_plain)
    assert np.array_equal(bits(got_s), bits(got_p)), np.flatnonzero(bits(got_s) != bits(got_p))[:8]
    orc, want, k_eff, _ = oracle.reduce([workloads.to_numpy(o) for o in objs], w.k, ORA_OP[op], ORA_DT[w.dtype],
                                        max(1, w.chunk_bytes // ES[w.dtype]), info_s["degree_used"], order, fm)
    assert orc == rc_s and info_s["k_eff"] == info_p["k_eff"] == k_eff
    assert np.array_equal(bits(got_s), bits(want))
    return info_s, info_p


def test_no_alloc_entry_point_equals_hop_reduce_on_two_calls_in_a_row():
    assert hop.hop_noalloc_scratch_bytes() == 8 << 20
    # many small objects (1000 inputs of 4 KiB, degree 16): the program as chains in one launch
    both_entry_points(workloads.WORKLOADS[5], "sum")
    # right after it a smaller call (fewer and shorter objects, ragged, a binary tree): whatever the first
    # call left in the scratch must not disturb it
    w = workloads.WORKLOADS[5].scaled(1024 + 12, 512, n=300, k=260, tree_degree=2, name="small_after_large")
    both_entry_points(w, "sum")
    both_entry_points(w, "max")


def test_no_alloc_long_program_large_objects_and_a_failure():
    # 150 steps over 2 MiB objects: too long for the kernel arguments, too large to be cut: the program
    # itself is staged in the scratch
    w = workloads.WORKLOADS[2].scaled(2 << 20, 256 << 10, n=200, k=150, tree_degree=4, name="staged_program")
    info_s, info_p = both_entry_points(w, "sum")
    assert info_s["n_launches"] == info_p["n_launches"] == 1
    # bf16 with a participant failing mid-stream: two launches, the second repairs the first
    w = workloads.WORKLOADS[4].scaled((1 << 20) + 6, 32 << 10)
    info_s, _ = both_entry_points(w, "sum", fm=w.fail_mask())
    assert info_s["k_eff"] == 31
    # hundreds of objects of 200 KiB: the one-launch form with 1 KiB columns, its table in the kernel arguments
    w = workloads.WORKLOADS[5].scaled(200 * 1024 + 8, 1 << 20, n=300, k=290, tree_degree=16, name="wide_columns", n_dst=0)
    info_s, info_p = both_entry_points(w, "sum")
    assert info_s["n_launches"] == info_p["n_launches"] == 1
    # thousands of objects of 3 KiB in a binary tree: no one-launch form; cut into sub-programs whose partial
    # results and records live in the static scratch
    w = workloads.WORKLOADS[5].scaled(3 * 1024 + 4, 4096, n=5000, k=5000, tree_degree=2, name="cut_in_scratch", n_dst=0)
    both_entry_points(w, "sum")
    # int32, short program (rides in the kernel arguments: no scratch at all)
    w = workloads.WORKLOADS[3].scaled(300 << 10, 16 << 10, n_dst=0)
    both_entry_points(w, "sum")


def test_no_alloc_rejects_what_does_not_fit():
    dev = torch.device("cuda:0")
    src = torch.ones(4, dtype=torch.float32, device=dev)
    dst = torch.full((4,), 7.0, dtype=torch.float32, device=dev)
    n = 600_000                                  # a chain over 600 000 inputs: 9.6 MB of program
    table = hop.PtrTable([int(src.data_ptr())] * n)
    rc, _ = hop.hop_reduce_noalloc(dst, table, n, "sum", "f32", 16, 1, object_bytes=16)
    torch.cuda.synchronize()
    assert rc == hop.HOP_ERR_TOO_LARGE and "scratch" in hop.hop_strerror(rc)
    assert torch.equal(dst.cpu(), torch.full((4,), 7.0))          # nothing was enqueued
    # and the next call works
    w = workloads.WORKLOADS[1]
    both_entry_points(w, "sum")


def test_no_alloc_call_over_many_small_objects_in_a_graph():
    # a call that allocates nothing and stages its tables through kernel arguments is nothing but kernel
    # launches: workload 5 (the program as chains, one launch behind the launches that carry its table)
    # recorded into a graph and replayed with other contents in the same buffers
    dev = torch.device("cuda:0")
    w = workloads.WORKLOADS[5]
    objs = workloads.make_objects(w, device=dev)
    order = w.ready_order()
    dst = torch.zeros_like(objs[0])
    rc, info = hop.hop_reduce_noalloc(dst, objs, w.k, "sum", w.dtype, w.chunk_bytes, w.tree_degree, order, None)
    torch.cuda.synchronize()
    assert rc == hop.HOP_OK
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        rc, info = hop.hop_reduce_noalloc(dst, objs, w.k, "sum", w.dtype, w.chunk_bytes, w.tree_degree, order, None)
    assert rc == hop.HOP_OK and info["n_launches"] == 1
    rng = np.random.default_rng(9)
    for rep in range(3):
        for o in objs[::37]:                          # eager work between the replays
            o.mul_(float(rng.uniform(0.5, 1.5)))
        dst.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        _, want, _, _ = oracle.reduce([workloads.to_numpy(o) for o in objs], w.k, oracle.SUM, oracle.F32,
                                      w.chunk_bytes // 4, w.tree_degree, order, None)
        assert np.array_equal(bits(workloads.to_numpy(dst)), bits(want)), rep
