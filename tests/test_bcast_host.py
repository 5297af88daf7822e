"""Receiver-driven broadcast coordination on the host (no GPU): the paper's worked example and
protocol invariants on random runs."""
import numpy as np
import pytest

import paper_2002_05814_amd as hop
from test_oracle_tree import read_golden

NAMES = {0: "S", 1: "R1", 2: "R2", 3: "R3"}


def edge(receiver, sender):
    return "%s<-%s" % (NAMES[receiver], NAMES[sender])


def test_fig4_sequence_without_failure():
    g = read_golden("fig4_broadcast_object.txt")
    C = 3                                           # three chunks, like the three elements of {5, 1, 0}
    rc, b = hop.hop_bcast_begin(None, 48, 16)
    assert rc == hop.HOP_OK and hop.hop_bcast_source_ready(b, C) == hop.HOP_OK
    r1, s1 = hop.hop_bcast_join(b)
    assert (r1, edge(r1, s1)) == (1, g["a"])
    assert hop.hop_bcast_step(b, 1) == hop.HOP_OK   # S has sent one chunk to R1 and is still busy
    r2, s2 = hop.hop_bcast_join(b)
    assert (r2, edge(r2, s2)) == (2, g["b"])
    hop.hop_bcast_step(b, 1)
    hop.hop_bcast_step(b, 1)                        # R1 now complete, still sending to R2; S is listed again
    assert hop.hop_bcast_sender(b, 1) == -1 and hop.hop_bcast_sender(b, 2) == 1
    r3, s3 = hop.hop_bcast_join(b)
    assert (r3, edge(r3, s3)) == (3, g["d"])        # complete S preferred over partial R2
    rc, info, log = hop.hop_bcast_finish(b)
    assert rc == hop.HOP_OK and info["n_complete"] == 3 and info["chunks_copied"] == 3 * C
    assert info["n_resumed"] == 0
    # every copy sent to at most one receiver at a time, and R2's chunks all came from R1
    assert {f for f, t, _, _ in log if t == 2} == {1} and {f for f, t, _, _ in log if t == 3} == {0}


def test_fig4_sequence_with_failure_of_r1():
    g = read_golden("fig4_broadcast_object.txt")
    C = 3
    rc, b = hop.hop_bcast_begin(None, 48, 16)
    hop.hop_bcast_source_ready(b, C)
    r1, _ = hop.hop_bcast_join(b)
    hop.hop_bcast_step(b, 1)
    r2, s2 = hop.hop_bcast_join(b)
    assert edge(r2, s2) == g["b"]
    hop.hop_bcast_step(b, 1)                        # R1 has 2 chunks, R2 has 1
    assert hop.hop_bcast_fail(b, r1) == hop.HOP_OK
    assert edge(r2, hop.hop_bcast_sender(b, r2)) == g["c_prime"]      # R2 resumes from S
    r3, s3 = hop.hop_bcast_join(b)
    assert edge(r3, s3) == g["d_prime"]             # S is busy with R2: R3 chains off R2
    rc, info, log = hop.hop_bcast_finish(b)
    assert rc == hop.HOP_OK and info["n_failed"] == 1 and info["n_resumed"] == 1 and info["n_complete"] == 2
    # R2 resumed where it was: chunk 0 from R1, chunks 1.. from S, nothing twice
    got = sorted((c0, c1, f) for f, t, c0, c1 in log if t == r2)
    assert got[0] == (0, 1, 1) and all(f == 0 for _, _, f in got[1:])
    assert sum(c1 - c0 for c0, c1, _ in got) == C


def check_log(log, n_copies, C, failed):
    """Protocol invariants from the log: chunks arrive in order, from a copy that already had them,
    and nothing is sent twice to the same receiver."""
    have = {0: C}
    for f, t, c0, c1 in log:
        assert 0 <= f < n_copies and 1 <= t < n_copies and f != t
        assert have.get(t, 0) == c0 and c0 < c1 <= C
        assert have.get(f, 0) >= c1
        have[t] = c1
    return have


def test_random_runs_keep_the_protocol_invariants():
    rng = np.random.default_rng(77)
    for it in range(200):
        C = int(rng.integers(1, 9))
        rc, b = hop.hop_bcast_begin(None, C * 32, 32)
        assert rc == hop.HOP_OK
        src_have, n_copies, failed = 0, 1, set()
        serving_now = {}
        for _ in range(int(rng.integers(1, 40))):
            what = rng.random()
            if what < 0.3 and src_have < C:
                src_have = min(C, src_have + int(rng.integers(1, 3)))
                assert hop.hop_bcast_source_ready(b, src_have) == hop.HOP_OK
            elif what < 0.55:
                rid, s = hop.hop_bcast_join(b)
                assert rid == n_copies and -1 <= s < rid and s not in failed
                n_copies += 1
            elif what < 0.62 and n_copies > 1:
                x = int(rng.integers(1, n_copies))
                assert hop.hop_bcast_fail(b, x) == hop.HOP_OK
                failed.add(x)
            else:
                assert hop.hop_bcast_step(b, int(rng.integers(0, 3))) == hop.HOP_OK
            # one receiver per sender at any time
            senders = [hop.hop_bcast_sender(b, i) for i in range(1, n_copies) if i not in failed]
            busy = [s for s in senders if s >= 0]
            assert len(busy) == len(set(busy)) and not (set(busy) & failed)
        hop.hop_bcast_source_ready(b, C)
        rc, info, log = hop.hop_bcast_finish(b)
        have = check_log(log, n_copies, C, failed)
        alive = [i for i in range(1, n_copies) if i not in failed]
        assert rc == hop.HOP_OK and info["n_complete"] == len(alive)
        assert all(have.get(i, 0) == C for i in alive)
        assert info["chunks_copied"] == sum(c1 - c0 for _, _, c0, c1 in log)
        assert info["n_receivers"] == n_copies - 1 and info["n_failed"] == len(failed)


def test_lost_original_leaves_receivers_partial():
    rc, b = hop.hop_bcast_begin(None, 4 * 32, 32)
    hop.hop_bcast_source_ready(b, 2)
    r1, s = hop.hop_bcast_join(b)
    hop.hop_bcast_step(b, 0)
    assert hop.hop_bcast_fail(b, 0) == hop.HOP_OK           # the only complete-to-be copy is gone
    rc, info, log = hop.hop_bcast_finish(b)
    assert rc == hop.HOP_PARTIAL and info["n_complete"] == 0
    assert hop.hop_bcast_begin(None, 64, 24)[0] == hop.HOP_ERR_INVALID
