"""Pins for the oracle's failure semantics (paper section 3.5.2)."""
import functools

import numpy as np
import pytest

import oracle

F32, BF16, I32 = oracle.F32, oracle.BF16, oracle.I32
SUM, MIN, MAX = oracle.SUM, oracle.MIN, oracle.MAX
TWO24 = float(2 ** 24)


def survivors_first_k(order, fm, C, k):
    alive = [int(i) for i in order if not (fm is not None and 0 <= fm[i] < C)]
    return alive[:k]


@pytest.mark.parametrize("d", [1, 2, 3, 8])
def test_int_result_is_reduce_over_first_k_survivors(d):
    rng = np.random.default_rng(40 + d)
    for _ in range(60):
        n = int(rng.integers(1, 11))
        k = int(rng.integers(1, n + 1))
        E, chunk = 24, 4                      # C = 6 chunks
        C = E // chunk
        objs = [rng.integers(-10 ** 6, 10 ** 6, size=E).astype(np.int32) for _ in range(n)]
        order = rng.permutation(n).astype(np.int32)
        fm = np.full(n, -1, np.int64)
        bad = rng.random(n) < 0.4
        fm[bad] = rng.integers(0, C + 2, size=int(bad.sum()))
        P = survivors_first_k(order, fm, C, k)
        for op, npop in ((SUM, np.add), (MIN, np.minimum), (MAX, np.maximum)):
            rc, dst, k_eff, _ = oracle.reduce(objs, k, op, I32, chunk, d, order, fm)
            if not P:
                assert rc == oracle.ERR_NO_SURVIVOR and dst is None
                continue
            assert rc == (oracle.OK if len(P) == k else oracle.PARTIAL) and k_eff == len(P)
            want = functools.reduce(npop, [objs[i].astype(np.int64) for i in P]).astype(np.int32)
            assert np.array_equal(dst, want)


@pytest.mark.parametrize("d", [1, 2, 4])
def test_result_does_not_depend_on_when_the_single_failure_happened(d):
    rng = np.random.default_rng(50 + d)
    n, k, E, chunk = 10, 6, 64, 8             # C = 8
    objs = [rng.standard_normal(E).astype(np.float32) for _ in range(n)]
    order = rng.permutation(n).astype(np.int32)
    for who in range(n):
        outs = []
        for c in range(1, 8):
            fm = np.full(n, -1, np.int64)
            fm[who] = c
            rc, dst, _, _ = oracle.reduce(objs, k, SUM, F32, chunk, d, order, fm)
            assert rc == oracle.OK
            outs.append(dst)
        assert all(np.array_equal(outs[0], o) for o in outs[1:])
        # c >= C: the object completed, so it did not fail at all
        fm = np.full(n, -1, np.int64)
        fm[who] = 8
        rc, dst, _, n_rep = oracle.reduce(objs, k, SUM, F32, chunk, d, order, fm)
        rc0, dst0, _, _ = oracle.reduce(objs, k, SUM, F32, chunk, d, order, None)
        assert n_rep == 0 and np.array_equal(dst, dst0)


def test_replacement_takes_the_failed_position_in_the_expression():
    # figure 5b: 6 of 10, R2 fails, R7 takes its place: (((R1+R7)+R3)+R4)+(R5+R6).
    # R1 = 2^24, R7 = 1, R3 = 1 -> (2^24+1)+1 = 2^24; if R7 were appended at the end instead,
    # grouped with nothing, the arithmetic would be the same here, so probe the pairing too:
    vals = [TWO24, 99.0, 1.0, 0.0, 0.0, 0.0, 1.0, 7.0, 7.0, 7.0]
    objs = [np.array([v], np.float32) for v in vals]
    fm = np.full(10, -1, np.int64)
    fm[1] = 3
    rc, dst, k_eff, n_rep = oracle.reduce(objs, 6, SUM, F32, 1, 2, None, fm)   # E=1, chunk=1 -> C=1 -> healthy
    assert n_rep == 0                                                          # c >= C means it completed
    objs8 = [np.full(8, v, np.float32) for v in vals]                          # C = 8 chunks of one element
    rc, dst, k_eff, n_rep = oracle.reduce(objs8, 6, SUM, F32, 1, 2, None, fm)
    assert rc == oracle.OK and n_rep == 1 and k_eff == 6
    assert np.all(dst == TWO24)                       # ((2^24 + 1) + 1) + 0 + (0 + 0): both ones absorbed
    # R5 = R6 = 1 instead: the right subtree still pairs them: 2^24 + 2
    vals2 = [TWO24, 99.0, 0.0, 0.0, 1.0, 1.0, 0.0, 7.0, 7.0, 7.0]
    objs8 = [np.full(8, v, np.float32) for v in vals2]
    rc, dst, _, _ = oracle.reduce(objs8, 6, SUM, F32, 1, 2, None, fm)
    assert np.all(dst == TWO24 + 2)
    # R7 = 1 and R3 = 1 with R1 = 0, R4 = 2^24: subtree {R1,R7,R3} sums to 2 before the root: 2^24 + 2
    vals3 = [0.0, 99.0, 1.0, TWO24, 0.0, 0.0, 1.0, 7.0, 7.0, 7.0]
    objs8 = [np.full(8, v, np.float32) for v in vals3]
    rc, dst, _, _ = oracle.reduce(objs8, 6, SUM, F32, 1, 2, None, fm)
    assert np.all(dst == TWO24 + 2)


def test_hole_keeps_the_tree_shape():
    # 6 of 6, R2 fails, nobody can replace it: ((R1 + R3) + R4) + (R5 + R6) with the right pair intact
    vals = [TWO24, 99.0, 0.0, 0.0, 1.0, 1.0]
    objs8 = [np.full(8, v, np.float32) for v in vals]
    fm = np.full(6, -1, np.int64)
    fm[1] = 5
    rc, dst, k_eff, n_rep = oracle.reduce(objs8, 6, SUM, F32, 1, 2, None, fm)
    assert rc == oracle.PARTIAL and k_eff == 5 and n_rep == 0
    assert np.all(dst == TWO24 + 2)      # a rebuilt 5-node tree would fold the ones in one by one: 2^24
    # a hole at the first position of a subtree: the next term starts the partial
    vals = [TWO24, 0.0, 0.0, 0.0, 99.0, 1.0]
    objs8 = [np.full(8, v, np.float32) for v in vals]
    fm = np.full(6, -1, np.int64)
    fm[4] = 2
    rc, dst, _, _ = oracle.reduce(objs8, 6, SUM, F32, 1, 2, None, fm)
    assert np.all(dst == TWO24)          # 2^24 + 1 -> 2^24
    # a whole subtree of holes contributes no term
    fm[5] = 1
    rc, dst, k_eff, _ = oracle.reduce(objs8, 6, SUM, F32, 1, 2, None, fm)
    assert k_eff == 4 and np.all(dst == TWO24)
    # chain with holes = left fold over the survivors in arrival order
    rng = np.random.default_rng(1)
    objs = [rng.standard_normal(16).astype(np.float32) for _ in range(7)]
    fm = np.full(7, -1, np.int64)
    fm[[2, 5]] = [1, 3]
    rc, dst, _, _ = oracle.reduce(objs, 7, SUM, F32, 2, 1, None, fm)
    want = functools.reduce(lambda a, b: (a + b).astype(np.float32), [objs[i] for i in (0, 1, 3, 4, 6)])
    assert np.array_equal(dst, want)


def test_failure_result_equals_clean_run_on_final_occupants():
    rng = np.random.default_rng(77)
    for _ in range(50):
        n = int(rng.integers(2, 12))
        k = int(rng.integers(1, n))
        d = int(rng.integers(1, 5))
        E, chunk = 32, 4
        objs = [rng.standard_normal(E).astype(np.float32) for _ in range(n)]
        order = rng.permutation(n).astype(np.int32)
        fm = np.full(n, -1, np.int64)
        bad = rng.choice(n, size=int(rng.integers(1, 3)), replace=False)
        fm[bad] = rng.integers(1, 8, size=len(bad))
        rc, occ, k_eff, _ = oracle.occupants(n, k, 8, order, fm)
        if rc != oracle.OK:
            continue
        rc, dst, _, _ = oracle.reduce(objs, k, SUM, F32, chunk, d, order, fm)
        rest = [i for i in range(n) if i not in set(occ.tolist())]
        clean_order = np.array(list(occ) + rest, np.int32)
        rc2, dst2, _, _ = oracle.reduce(objs, k, SUM, F32, chunk, d, clean_order, None)
        assert rc == rc2 == oracle.OK and np.array_equal(dst, dst2)
