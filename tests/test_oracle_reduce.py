"""Pins for the oracle's arithmetic and association order.

Expected values come from closed forms, from textbook left folds written with
numpy scalars, from library routines (numpy reductions, torch's bfloat16
conversion) and from hand-built rounding probes whose result reveals how the
terms were grouped; never from the oracle itself.
"""
import functools

import numpy as np
import pytest
import torch

import oracle
import workloads

F32, BF16, I32 = oracle.F32, oracle.BF16, oracle.I32
SUM, MIN, MAX = oracle.SUM, oracle.MIN, oracle.MAX
TWO24 = float(2 ** 24)


def f32(*vals):
    return [np.array([v], np.float32) for v in vals]


def run(objs, k=None, op=SUM, dtype=F32, d=2, order=None, fm=None, chunk=1 << 30):
    rc, dst, k_eff, n_rep = oracle.reduce(objs, len(objs) if k is None else k, op, dtype, chunk, d, order, fm)
    assert rc >= 0, rc
    return dst


# ------------------------------------------------------------ grouping probes (figure 5a)

def test_subtree_partials_are_formed_before_meeting_the_root():
    # k = 6, d = 2, arrivals a0..a5 = R1..R6. R2 reduces {R1,R2,R3} before R4 adds it.
    # 0.5+0.5+0.5 = 1.5 and 2^24 + 1.5 rounds to 2^24 + 2, whereas adding the halves to 2^24
    # one by one leaves 2^24 (each 0.5 is below half an ulp).
    got = run(f32(0.5, 0.5, 0.5, TWO24, 0.0, 0.0), d=2)
    assert got[0] == TWO24 + 2
    # R6 reduces {R5,R6} before the root sees them: 2^24 + (1+1) = 2^24+2, but
    # (2^24 + 1) + 1 = 2^24 under round-to-nearest-even.
    got = run(f32(TWO24, 0.0, 0.0, 0.0, 1.0, 1.0), d=2)
    assert got[0] == TWO24 + 2
    # a chain (d=1) is a plain left fold: the same inputs lose both ones
    got = run(f32(TWO24, 0.0, 0.0, 0.0, 1.0, 1.0), d=1)
    assert got[0] == TWO24
    # and so does the star (d >= k-1)
    got = run(f32(TWO24, 0.0, 0.0, 0.0, 1.0, 1.0), d=5)
    assert got[0] == TWO24


def test_node_combines_first_child_then_self_then_other_children():
    # k = 3, d = 2: arrivals a0 (first child), a1 (root), a2 (second child): (a0 + a1) + a2.
    # With a0 = 2^24, a1 = 1, a2 = 1 -> ((2^24+1)+1) = 2^24; any order that pairs the ones gives 2^24+2.
    assert run(f32(TWO24, 1.0, 1.0), d=2)[0] == TWO24
    # a0 = 1, a1 = 1, a2 = 2^24: (1+1)+2^24 = 2^24+2; a grouping that adds a2 earlier gives 2^24
    assert run(f32(1.0, 1.0, TWO24), d=2)[0] == TWO24 + 2
    # k = 4, d = 3: arrivals: first child, root, second child, third child: ((a0+a1)+a2)+a3
    assert run(f32(1.0, 1.0, TWO24, 0.0), d=3)[0] == TWO24 + 2
    assert run(f32(TWO24, 1.0, 1.0, 1.0), d=3)[0] == TWO24
    # ((1+1)+2^24)+1 = 2^24+3 -> tie -> even mantissa = 2^24+4
    assert run(f32(1.0, 1.0, TWO24, 1.0), d=3)[0] == TWO24 + 4


def test_parenthesisation_of_the_two_headline_trees():
    # the grouping the definition gives for k = 8, d = 2 and k = 12, d = 4, written out by hand with
    # numpy float32 adds (values with wildly different magnitudes so that every grouping differs)
    rng = np.random.default_rng(33)
    a = [(rng.standard_normal(64) * 10.0 ** rng.integers(-4, 5, size=64)).astype(np.float32) for _ in range(12)]
    f = np.float32

    def add(x, y):
        return (x + y).astype(f)
    # k = 8, d = 2: ((((a0+a1)+a2)+a3)+a4) + ((a5+a6)+a7)
    want8 = add(add(add(add(add(a[0], a[1]), a[2]), a[3]), a[4]), add(add(a[5], a[6]), a[7]))
    assert np.array_equal(run(a[:8], d=2), want8)
    # k = 12, d = 4: L = (((a0+a1)+a2)+a3)+a4, M = ((a6+a7)+a8)+a9, result (((L+a5)+M)+a10)+a11
    L = add(add(add(add(a[0], a[1]), a[2]), a[3]), a[4])
    M = add(add(add(a[6], a[7]), a[8]), a[9])
    want12 = add(add(add(add(L, a[5]), M), a[10]), a[11])
    assert np.array_equal(run(a, d=4), want12)
    # and they are not the plain left fold
    fold = functools.reduce(add, a)
    assert not np.array_equal(want12, fold)


def test_min_max_keep_the_earlier_term_on_ties():
    # the comparison forms keep the left operand unless the right one is strictly better, and a node
    # combines [first child, itself, second child] left to right: with -0.0 and +0.0 (equal under
    # comparison) the sign of the result names the term that came first
    neg0, pos0 = np.float32(-0.0), np.float32(0.0)
    for op in (MAX, MIN):
        got = run([np.array([neg0]), np.array([pos0]), np.array([pos0])], op=op, d=2)
        assert np.signbit(got[0])                  # first child (-0.0) came first
        got = run([np.array([pos0]), np.array([neg0]), np.array([neg0])], op=op, d=2)
        assert not np.signbit(got[0])
        got = run([np.array([pos0]), np.array([neg0])], op=op, d=1)
        assert not np.signbit(got[0])


def test_ready_order_decides_position_not_object_index():
    objs = f32(1.0, TWO24, 1.0)          # object 1 is the big one
    # arrival order 0,2,1 -> (1+1)+2^24
    assert run(objs, d=2, order=[0, 2, 1])[0] == TWO24 + 2
    # arrival order 1,0,2 -> (2^24+1)+1
    assert run(objs, d=2, order=[1, 0, 2])[0] == TWO24


# ------------------------------------------------------------ degenerate shapes = textbook left fold

@pytest.mark.parametrize("d", [1, 10 ** 6])
@pytest.mark.parametrize("k", [1, 2, 3, 7, 33])
def test_chain_and_star_equal_numpy_left_fold(k, d):
    rng = np.random.default_rng(k * 7 + (d > 1))
    n = k + 3
    objs = [rng.standard_normal(257).astype(np.float32) * np.float32(10.0 ** rng.integers(-3, 4)) for _ in range(n)]
    order = rng.permutation(n).astype(np.int32)
    got = run(objs, k=k, d=max(d, 1), order=order)
    want = functools.reduce(lambda a, b: (a + b).astype(np.float32), [objs[i] for i in order[:k]])
    assert got.dtype == np.float32 and np.array_equal(got, want)


# ------------------------------------------------------------ order-free cases: closed forms / library

@pytest.mark.parametrize("d", [1, 2, 3, 4, 8, 16, 1000])
def test_exactly_summable_floats_equal_integer_sum(d):
    # multiples of 2^-6 with |m| < 2^17: every partial sum of up to 64 terms is exact in binary32,
    # so every association order must give the integer sum
    rng = np.random.default_rng(d)
    n, k, E = 64, 50, 300
    m = rng.integers(-(1 << 17) + 1, 1 << 17, size=(n, E))
    objs = [(m[i] * 2.0 ** -6).astype(np.float32) for i in range(n)]
    order = rng.permutation(n).astype(np.int32)
    got = run(objs, k=k, d=d, order=order)
    want = (m[order[:k]].sum(axis=0) * 2.0 ** -6)
    assert np.array_equal(got.astype(np.float64), want)


@pytest.mark.parametrize("dtype", [F32, I32, BF16])
@pytest.mark.parametrize("d", [1, 2, 4, 16])
def test_identical_objects(dtype, d):
    k = 24
    if dtype == I32:
        x = np.array([0, 1, -1, 123456789, -2 ** 31, 2 ** 31 - 1, 2 ** 30], np.int32)
        want = ((x.astype(np.int64) * k + 2 ** 31) % 2 ** 32 - 2 ** 31).astype(np.int32)   # wraps mod 2^32
    elif dtype == F32:
        x = np.array([0.0, 1.0, -3.0, 0.375, 1024.0, -2.0 ** -20], np.float32)
        want = (x * np.float32(k)).astype(np.float32)        # k*x exact for these values
    else:
        xf = np.array([0.0, 1.0, -3.0, 0.375, 96.0, -2.0 ** -20], np.float32)
        x = (xf.view(np.uint32) >> 16).astype(np.uint16)      # exactly representable in bf16
        want = ((xf * np.float32(k)).view(np.uint32) >> 16).astype(np.uint16)   # 24*x still has <= 8 significant bits
    objs = [x.copy() for _ in range(k + 2)]
    for op, w in ((SUM, want), (MIN, x), (MAX, x)):           # min/max idempotent
        got = run(objs, k=k, op=op, dtype=dtype, d=d)
        assert np.array_equal(got, w), (op, dtype)


@pytest.mark.parametrize("d", [1, 2, 3, 8])
def test_int32_sum_min_max_against_numpy(d):
    rng = np.random.default_rng(100 + d)
    n, k, E = 20, 13, 1000
    objs = [rng.integers(-2 ** 31, 2 ** 31, size=E, dtype=np.int64).astype(np.int32) for _ in range(n)]
    order = rng.permutation(n).astype(np.int32)
    P = np.stack([objs[i] for i in order[:k]])
    want_sum = ((P.astype(np.int64).sum(axis=0) + 2 ** 31) % 2 ** 32 - 2 ** 31).astype(np.int32)
    assert np.array_equal(run(objs, k=k, op=SUM, dtype=I32, d=d, order=order), want_sum)
    assert np.array_equal(run(objs, k=k, op=MIN, dtype=I32, d=d, order=order), P.min(axis=0))
    assert np.array_equal(run(objs, k=k, op=MAX, dtype=I32, d=d, order=order), P.max(axis=0))
    # integer results do not depend on the order in which the same k objects arrived
    order2 = np.concatenate([rng.permutation(order[:k]), order[k:]]).astype(np.int32)
    assert np.array_equal(run(objs, k=k, op=SUM, dtype=I32, d=d, order=order2), want_sum)


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("d", [1, 2, 4, 16])
def test_float_min_max_against_numpy(dtype, d):
    rng = np.random.default_rng(200 + d)
    n, k, E = 17, 11, 513
    vals = [rng.standard_normal(E).astype(np.float32) for _ in range(n)]
    if dtype == BF16:
        vals = [(v.view(np.uint32) & 0xFFFF0000).view(np.float32) for v in vals]
        objs = [(v.view(np.uint32) >> 16).astype(np.uint16) for v in vals]
    else:
        objs = vals
    order = rng.permutation(n).astype(np.int32)
    P = np.stack([vals[i] for i in order[:k]])
    for op, want in ((MAX, P.max(axis=0)), (MIN, P.min(axis=0))):
        got = run(objs, k=k, op=op, dtype=dtype, d=d, order=order)
        if dtype == BF16:
            got = (got.astype(np.uint32) << 16).view(np.float32)
        assert np.array_equal(got, want)
    # min(x) = -max(-x)
    neg = [(-v) for v in vals]
    nobjs = neg if dtype == F32 else [(v.view(np.uint32) >> 16).astype(np.uint16) for v in neg]
    a = run(objs, k=k, op=MIN, dtype=dtype, d=d, order=order)
    b = run(nobjs, k=k, op=MAX, dtype=dtype, d=d, order=order)
    if dtype == BF16:
        a = (a.astype(np.uint32) << 16).view(np.float32)
        b = (b.astype(np.uint32) << 16).view(np.float32)
    assert np.array_equal(a, -b)


def test_once_and_only_once_one_hot():
    # object i is 1 at element i and 0 elsewhere: the sum is the indicator of who was folded in
    n, k = 12, 7
    order = np.random.default_rng(3).permutation(n).astype(np.int32)
    objs = [np.eye(n, dtype=np.int32)[i] for i in range(n)]
    for d in (1, 2, 3, 12):
        got = run(objs, k=k, dtype=I32, d=d, order=order)
        want = np.zeros(n, np.int32)
        want[order[:k]] = 1
        assert np.array_equal(got, want)


# ------------------------------------------------------------ free-order tolerance vs float64

@pytest.mark.parametrize("d", [1, 2, 4, 8])
def test_f32_sum_close_to_float64_and_to_reduce_set(d):
    rng = np.random.default_rng(300 + d)
    n, k, E = 40, 32, 2000
    objs = [rng.standard_normal(E).astype(np.float32) for _ in range(n)]
    order = rng.permutation(n).astype(np.int32)
    got = run(objs, k=k, d=d, order=order).astype(np.float64)
    P = np.stack([objs[i] for i in order[:k]]).astype(np.float64)
    want = P.sum(axis=0)
    scale = np.maximum(np.abs(want), np.abs(P).sum(axis=0) / k)
    assert np.all(np.abs(got - want) <= 1e-5 * np.log2(k) * scale)
    rc, occ, _, _ = oracle.occupants(n, k, 1, order, None)
    ref = oracle.reduce_set(objs, occ, SUM, F32)
    assert np.allclose(ref, want, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("op,np_red", [(SUM, None), (MIN, np.minimum), (MAX, np.maximum)])
def test_reduce_set_every_branch_against_library_reductions(op, np_red):
    # the order-free definition in every element type and op, with empty positions (-1) among the
    # occupants: int32 carried in int64 (the sum leaves the int32 range and must not wrap), floats in
    # float64; expected values from numpy's int64 / float64 reductions, math.fsum (exact) and torch's
    # bfloat16 widening
    import math
    rng = np.random.default_rng(40 + op)
    n, E = 20, 600
    occ = np.array([3, -1, 17, 0, 9, -1, 12, 5, 19, 1], np.int32)        # two empty positions
    live = [int(o) for o in occ if o >= 0]
    # int32: values near the ends of the range
    ints = [rng.integers(-2 ** 31, 2 ** 31, size=E, dtype=np.int64).astype(np.int32) for _ in range(n)]
    for i in live:
        ints[i][:8] = np.int32(2 ** 31 - 1)
    got = oracle.reduce_set(ints, occ, op, I32)
    P = np.stack([ints[i] for i in live]).astype(np.int64)
    want = P.sum(axis=0) if op == SUM else np_red.reduce(P, axis=0)
    assert got.dtype == np.int64 and np.array_equal(got, want)
    if op == SUM:
        assert got[0] > 2 ** 32                      # really unwrapped
    # float32
    flts = [(rng.standard_normal(E) * 10.0 ** rng.integers(-4, 5)).astype(np.float32) for _ in range(n)]
    got = oracle.reduce_set(flts, occ, op, F32)
    Pf = np.stack([flts[i] for i in live]).astype(np.float64)
    if op == SUM:
        exact = np.array([math.fsum(Pf[:, e]) for e in range(E)])
        assert np.all(np.abs(got - exact) <= 1e-15 * np.abs(Pf).sum(axis=0) * len(live))
    else:
        assert np.array_equal(got, np_red.reduce(Pf, axis=0))
    # bfloat16 (bit patterns), widened by torch
    halves = [rng.integers(0, 1 << 16, size=E, dtype=np.uint32).astype(np.uint16) for _ in range(n)]
    for h in halves:
        h[(h & 0x7F80) == 0x7F80] = 0x3F80          # no infinities or NaNs among the inputs
    wide = [torch.from_numpy(h.view(np.int16).copy()).view(torch.bfloat16).double().numpy() for h in halves]
    got = oracle.reduce_set(halves, occ, op, BF16)
    Pb = np.stack([wide[i] for i in live])
    if op == SUM:
        exact = np.array([math.fsum(Pb[:, e]) for e in range(E)])
        assert np.all(np.abs(got - exact) <= 1e-15 * np.abs(Pb).sum(axis=0) * len(live))
    else:
        assert np.array_equal(got, np_red.reduce(Pb, axis=0))
    # a single occupant comes back unchanged, whatever the op
    one = np.array([-1, 7, -1], np.int32)
    assert np.array_equal(oracle.reduce_set(flts, one, op, F32), flts[7].astype(np.float64))
    assert np.array_equal(oracle.reduce_set(ints, one, op, I32), ints[7].astype(np.int64))


# ------------------------------------------------------------ bfloat16

def test_bf16_conversion_matches_torch_exhaustively():
    hi = np.arange(1 << 16, dtype=np.uint32) << 16
    for lo in (0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF):
        bits = (hi | np.uint32(lo)).astype(np.uint32)
        x = bits.view(np.float32)
        got = oracle.f32_to_bf16(x)
        want = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        nan = np.isnan(x)
        assert np.array_equal(got[~nan], want[~nan]), hex(lo)
        # NaN stays NaN
        assert np.all(np.isnan((got[nan].astype(np.uint32) << 16).view(np.float32)))
    # widening is exact
    h = np.arange(1 << 16, dtype=np.uint16)
    w = oracle.bf16_to_f32(h)
    assert np.array_equal(w.view(np.uint32), h.astype(np.uint32) << 16)


@pytest.mark.parametrize("d", [1, 1000])
def test_bf16_sum_accumulates_in_f32_and_rounds_once(d):
    # left fold in float32 of the widened inputs, one final conversion: written with torch
    rng = np.random.default_rng(17 + d)
    n, k, E = 40, 33, 700
    ts = [torch.from_numpy(rng.standard_normal(E).astype(np.float32)).to(torch.bfloat16) for _ in range(n)]
    objs = [workloads.to_numpy(t) for t in ts]
    order = rng.permutation(n).astype(np.int32)
    acc = ts[order[0]].to(torch.float32)
    for i in order[1:k]:
        acc = acc + ts[i].to(torch.float32)
    want = workloads.to_numpy(acc.to(torch.bfloat16))
    got = run(objs, k=k, dtype=BF16, d=d, order=order)
    assert np.array_equal(got, want)
    # rounding after every add (a bf16 accumulator) would differ: the test can tell the two apart
    acc16 = ts[order[0]].clone()
    for i in order[1:k]:
        acc16 = (acc16.to(torch.float32) + ts[i].to(torch.float32)).to(torch.bfloat16)
    assert not np.array_equal(workloads.to_numpy(acc16), want)


# ------------------------------------------------------------ broadcast / allreduce

def test_broadcast_paper_example_and_bytes():
    import os
    from test_oracle_tree import read_golden
    g = read_golden("fig4_broadcast_object.txt")
    src = np.array([int(v) for v in g["object"].split()], np.int32)
    outs = oracle.broadcast(src, len(g["receivers"].split()))
    assert len(outs) == 3 and all(o.tolist() == [5, 1, 0] for o in outs)
    blob = np.frombuffer(os.urandom(1000), np.uint8)
    for o in oracle.broadcast(blob, 5):
        assert o.tobytes() == blob.tobytes()
    assert oracle.broadcast(blob, 0) == []


def test_allreduce_is_reduce_then_broadcast():
    rng = np.random.default_rng(9)
    objs = [rng.integers(-1000, 1000, size=64).astype(np.int32) for _ in range(6)]
    rc, outs, k_eff, _ = oracle.allreduce(objs, 4, 6, SUM, I32, 16, 2)
    want = np.stack(objs).sum(axis=0).astype(np.int32)
    assert rc == oracle.OK and len(outs) == 4 and all(np.array_equal(o, want) for o in outs)


# ------------------------------------------------------------ workload structure

def test_softmax_workload_mass_is_k_eff():
    w = workloads.WORKLOADS[5]
    objs = [workloads.to_numpy(t) for t in workloads.make_objects(w)]
    order = w.ready_order()
    rc, dst, k_eff, _ = oracle.reduce(objs, w.k, SUM, F32, w.chunk_bytes // 4, w.tree_degree, order, None)
    assert rc == oracle.OK and k_eff == 1000
    assert abs(float(dst.astype(np.float64).sum()) - 1000.0) < 1e-2     # every object sums to 1
    rc, mx, _, _ = oracle.reduce(objs, w.k, MAX, F32, w.chunk_bytes // 4, w.tree_degree, order, None)
    assert np.all(mx > 0) and np.all(mx <= 1)
    assert np.array_equal(mx, np.stack([objs[i] for i in order[:w.k]]).max(axis=0))
