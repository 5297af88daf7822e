"""Pins for the oracle's tree shape, slot numbering and occupant rules.

None of these re-derive the oracle's own code: they check it against the
paper's worked example (tests/golden/fig5_reduce_tree.txt), against properties
an in-order numbering must have, and against brute-force set arithmetic.
"""
import itertools
import math
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, val = line.split("=", 1)
            out[key.strip()] = val.strip()
    return out


def children(j, d, k):
    return [d * j + c for c in range(1, d + 1) if d * j + c < k]


def subtree_nodes(j, d, k):
    out = [j]
    for c in children(j, d, k):
        out += subtree_nodes(c, d, k)
    return out


def ancestors(j, par):
    out = []
    while par[j] >= 0:
        j = par[j]
        out.append(j)
    return out


# ---------------------------------------------------------------- paper example

def test_fig5_worked_example():
    g = read_golden("fig5_reduce_tree.txt")
    k, d = int(g["k"]), int(g["d"])
    names = g["arrival"].split()
    nos, par = oracle.tree_slots(k, d)
    node_of = {names[t]: int(nos[t]) for t in range(k)}
    name_of = {v: n for n, v in node_of.items()}
    # root is the 4th arrival
    assert par[node_of[g["root"]]] == -1
    # R2's only ancestor is R4
    assert [name_of[a] for a in ancestors(node_of["R2"], par)] == g["ancestors_of_R2"].split()
    # subtrees named by the figure's description
    assert sorted(name_of[j] for j in subtree_nodes(node_of["R2"], d, k)) == sorted(g["subtree_of_R2"].split())
    assert sorted(name_of[j] for j in subtree_nodes(node_of["R6"], d, k)) == sorted(g["subtree_of_R6"].split())


def test_fig5_failure_replacement():
    g = read_golden("fig5_reduce_tree.txt")
    k, n = int(g["k"]), int(g["n_sources"])
    # objects R1..R10 are indices 0..9 and arrive in that order; R2 fails mid-stream
    C = 8
    for c_fail in range(1, C):
        fm = np.full(n, -1, np.int64)
        fm[1] = c_fail
        rc, occ, k_eff, n_rep = oracle.occupants(n, k, C, None, fm)
        assert rc == oracle.OK and k_eff == k and n_rep == 1
        final = sorted("R%d" % (i + 1) for i in occ)
        assert final == sorted(g["final_set"].split())
        # R7 (index 6) sits where R2 was: slot 1 (second arrival)
        assert occ[1] == 6
        # everyone else kept their place
        assert [occ[t] for t in (0, 2, 3, 4, 5)] == [0, 2, 3, 4, 5]


def test_six_of_ten_takes_earliest_six():
    rng = np.random.default_rng(7)
    for _ in range(20):
        order = rng.permutation(10).astype(np.int32)
        rc, occ, k_eff, n_rep = oracle.occupants(10, 6, 4, order, None)
        assert rc == oracle.OK and k_eff == 6 and n_rep == 0
        assert list(occ) == list(order[:6])


# ---------------------------------------------------------------- in-order properties

@pytest.mark.parametrize("k,d", [(k, d) for k in range(1, 41) for d in (1, 2, 3, 4, 8, 16, 64)])
def test_inorder_numbering_properties(k, d):
    nos, par = oracle.tree_slots(k, d)
    # a permutation of the nodes
    assert sorted(nos.tolist()) == list(range(k))
    slot = {int(nos[t]): t for t in range(k)}
    for j in range(k):
        ch = children(j, d, k)
        for c in ch:
            assert par[c] == j
        # every subtree occupies a contiguous run of arrival slots ...
        s = sorted(slot[x] for x in subtree_nodes(j, d, k))
        assert s == list(range(s[0], s[0] + len(s)))
        # ... first child's subtree entirely before the node, the others after, left to right
        if ch:
            assert max(slot[x] for x in subtree_nodes(ch[0], d, k)) == slot[j] - 1
            prev = slot[j]
            for c in ch[1:]:
                cs = sorted(slot[x] for x in subtree_nodes(c, d, k))
                assert cs[0] == prev + 1
                prev = cs[-1]
    # "at most log_d n nodes clear": no slot has more ancestors than the height of a
    # complete d-ary tree on k nodes
    if d >= 2:
        height = 0
        while (d ** (height + 1) - 1) // (d - 1) < k:
            height += 1
        assert max(len(ancestors(j, par)) for j in range(k)) == height
        assert height <= math.ceil(math.log(max(k, 2), d)) + 0
    else:
        assert max(len(ancestors(j, par)) for j in range(k)) == k - 1


def test_chain_and_star_shapes():
    # d = 1: a single chain, arrival t sits k-1-t levels above the first arrival
    nos, par = oracle.tree_slots(7, 1)
    assert nos.tolist() == [6, 5, 4, 3, 2, 1, 0]
    # d >= k-1: a root connected to everyone; first arrival is its first child,
    # the root is the second arrival, the rest follow in order
    for d in (6, 7, 100, 2 ** 30):
        nos, par = oracle.tree_slots(7, d)
        assert nos.tolist() == [1, 0, 2, 3, 4, 5, 6]
        assert par.tolist() == [-1, 0, 0, 0, 0, 0, 0]


# ---------------------------------------------------------------- occupants: brute force on sets

def brute_first_k_survivors(n, k, C, order, fm):
    """Section 3.5.2 as a set statement: the first k ready objects that do not fail."""
    alive = []
    for i in order:
        c = -1 if fm is None else fm[i]
        if 0 <= c < C:
            continue
        alive.append(int(i))
    return set(alive[:k])


def test_occupant_set_equals_first_k_survivors_exhaustive_single_failure():
    C = 3
    for n in range(1, 8):
        for k in range(1, n + 1):
            order = np.random.default_rng(n * 10 + k).permutation(n).astype(np.int32)
            for who in range(n):
                for c in range(0, C + 2):
                    fm = np.full(n, -1, np.int64)
                    fm[who] = c
                    rc, occ, k_eff, _ = oracle.occupants(n, k, C, order, fm)
                    want = brute_first_k_survivors(n, k, C, order, fm)
                    if not want:
                        assert rc == oracle.ERR_NO_SURVIVOR
                        continue
                    got = [int(x) for x in occ if x >= 0]
                    assert len(got) == len(set(got))              # once and only once
                    assert set(got) == want
                    assert k_eff == len(want)
                    assert rc == (oracle.OK if len(want) == k else oracle.PARTIAL)


def test_occupant_set_random_multi_failure():
    rng = np.random.default_rng(11)
    for _ in range(400):
        n = int(rng.integers(1, 12))
        k = int(rng.integers(1, n + 1))
        C = int(rng.integers(1, 6))
        order = rng.permutation(n).astype(np.int32)
        fm = rng.integers(-1, C + 2, size=n).astype(np.int64)
        fm[rng.random(n) < 0.5] = -1
        rc, occ, k_eff, _ = oracle.occupants(n, k, C, order, fm)
        want = brute_first_k_survivors(n, k, C, order, fm)
        if not want:
            assert rc == oracle.ERR_NO_SURVIVOR
            continue
        got = [int(x) for x in occ if x >= 0]
        assert len(got) == len(set(got)) and set(got) == want and k_eff == len(want)


def test_survivors_keep_their_slots():
    # well-behaving participants are never moved: a healthy initial slot holder stays put
    rng = np.random.default_rng(5)
    for _ in range(200):
        n = int(rng.integers(2, 12))
        k = int(rng.integers(1, n + 1))
        C = 4
        order = rng.permutation(n).astype(np.int32)
        fm = np.full(n, -1, np.int64)
        bad = rng.choice(n, size=int(rng.integers(1, n)), replace=False)
        fm[bad] = rng.integers(1, C, size=len(bad))
        rc, occ, _, _ = oracle.occupants(n, k, C, order, fm)
        for t in range(k):
            if fm[order[t]] < 0:
                assert occ[t] == order[t]


def test_failure_order_is_time_order():
    # two slot holders fail; the one that fails earlier (fewer chunks delivered) gets
    # the first waiting object, whichever slot it holds
    n, k, C = 6, 4, 8
    fm = np.full(n, -1, np.int64)
    fm[0], fm[2] = 5, 2            # slot 0 fails late, slot 2 fails early
    rc, occ, _, n_rep = oracle.occupants(n, k, C, None, fm)
    assert rc == oracle.OK and n_rep == 2
    assert occ.tolist() == [5, 1, 4, 3]
    # same time: ascending arrival (slot) order
    fm[0], fm[2] = 3, 3
    rc, occ, _, _ = oracle.occupants(n, k, C, None, fm)
    assert occ.tolist() == [4, 1, 5, 3]


def test_never_ready_holds_no_slot_and_dead_pool_member_is_skipped():
    n, k, C = 6, 3, 4
    fm = np.full(n, -1, np.int64)
    fm[1] = 0                       # never becomes ready: skipped in the ready order
    rc, occ, k_eff, n_rep = oracle.occupants(n, k, C, None, fm)
    assert occ.tolist() == [0, 2, 3] and n_rep == 0 and rc == oracle.OK
    fm[4] = 1                       # pool member dies early
    fm[0] = 2                       # slot holder dies later: replacement must skip object 4
    rc, occ, k_eff, n_rep = oracle.occupants(n, k, C, None, fm)
    assert occ.tolist() == [5, 2, 3] and n_rep == 1
    # a replacement that itself fails later is replaced again, or leaves a hole
    fm = np.full(n, -1, np.int64)
    fm[0], fm[3] = 1, 2
    rc, occ, k_eff, n_rep = oracle.occupants(n, 3, C, None, fm)
    assert occ.tolist() == [4, 1, 2] and n_rep == 2
    fm = np.full(4, -1, np.int64)
    fm[0], fm[3] = 1, 2
    rc, occ, k_eff, n_rep = oracle.occupants(4, 3, C, None, fm)
    assert occ.tolist() == [-1, 1, 2] and rc == oracle.PARTIAL and k_eff == 2


def test_invalid_arguments():
    assert oracle.occupants(4, 5, 2, None, None)[0] == oracle.ERR_INVALID
    assert oracle.occupants(4, 2, 2, np.array([0, 1, 1, 3], np.int32), None)[0] == oracle.ERR_INVALID
    assert oracle.occupants(4, 2, 2, np.array([0, 1, 2, 4], np.int32), None)[0] == oracle.ERR_INVALID
    with pytest.raises(ValueError):
        oracle.tree_slots(0, 2)
    with pytest.raises(ValueError):
        oracle.tree_slots(3, 0)
