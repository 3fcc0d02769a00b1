"""Pins for the oracle's most-recent-neighbour sampler (Sec. 2.1 "most recent neighbors"): neighbour lists
written out by hand, a pure-Python walk over the event list, the strict-past invariant, and the indexed form
(used on graphs too long to scan per query) against the scan."""
import numpy as np
import pytest

from oracle import tgnn_oracle as O


def brute_force(src, dst, ts, node, t, k):
    """Walk all events; keep those touching `node` with time < t; order by (time, id); take last k."""
    cand = []
    for e in range(len(src)):
        if ts[e] < t:
            if src[e] == node:
                cand.append((ts[e], e, dst[e]))
            if dst[e] == node:
                cand.append((ts[e], e, src[e]))
    cand.sort(key=lambda c: (c[0], c[1]))
    return cand[::-1][:k]


def test_hand_written_lists():
    """Six events, written out; the expected rows are read off this table by eye.
         id  0      1      2      3      4      5
         u-v 0-1    2-0    0-1    3-0    1-2    0-3
         t   1.0    2.0    2.0    4.0    5.0    5.0"""
    src = np.array([0, 2, 0, 3, 1, 0]); dst = np.array([1, 0, 1, 0, 2, 3])
    ts = np.array([1.0, 2.0, 2.0, 4.0, 5.0, 5.0])
    qn = np.array([0, 0, 0, 1, 2, 3, 0])
    qt = np.array([5.0, 2.0, 9.0, 5.0, 2.0, 4.5, 0.5])
    nbr, ne, nts, cnt = O.sample_recent(src, dst, ts, qn, qt, 3)
    assert cnt.tolist() == [3, 1, 3, 2, 0, 1, 0]
    # node 0 before t = 5: events 0, 1, 2, 3 (event 5 at t = 5 is not earlier); last three, most recent first
    assert ne[0].tolist() == [3, 2, 1] and nbr[0].tolist() == [3, 1, 2] and nts[0].tolist() == [4.0, 2.0, 2.0]
    # node 0 before t = 2: only event 0 (the two events at t = 2 are not strictly earlier)
    assert ne[1].tolist() == [0, -1, -1] and nbr[1].tolist() == [1, -1, -1] and nts[1].tolist() == [1.0, 0.0, 0.0]
    # node 0 before t = 9: all five of its events; the last three are 5, 3, 2
    assert ne[2].tolist() == [5, 3, 2] and nbr[2].tolist() == [3, 3, 1]
    # node 1 before t = 5: events 0 and 2 (event 4 at t = 5 excluded); equal-time tie at t = 2 resolved by id above
    assert ne[3].tolist() == [2, 0, -1] and nbr[3].tolist() == [0, 0, -1]
    # node 2 before t = 2: its first event is at t = 2 -> nothing
    assert ne[4].tolist() == [-1, -1, -1]
    # node 3 before t = 4.5: event 3 (as its source: the other endpoint is the destination 0)
    assert ne[5].tolist() == [3, -1, -1] and nbr[5].tolist() == [0, -1, -1]


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_scan_and_indexed_form_vs_python_walk_with_ties(seed):
    rng = np.random.default_rng(seed)
    n, E, k = 30, 400, 5
    src = rng.integers(0, n - 3, E); dst = rng.integers(0, n - 3, E)      # nodes n-3.. have no events; self loops occur
    ts = np.sort(rng.integers(0, 60, E)).astype(np.float64)               # many equal timestamps
    assert np.any(src == dst)
    qn = rng.integers(0, n, 300); qt = rng.integers(-1, 62, 300).astype(np.float64)
    scan = O.sample_recent(src, dst, ts, qn, qt, k)
    indexed = O.sample_recent_indexed(O.build_adjacency(src, dst, ts, n), qn, qt, k)
    for a, b in zip(scan, indexed):
        assert np.array_equal(a, b)
    nbr, ne, nts, cnt = scan
    for r in range(len(qn)):
        ref = brute_force(src, dst, ts, qn[r], qt[r], k)
        assert cnt[r] == len(ref)
        for j, (tt, e, other) in enumerate(ref):
            assert (nbr[r, j], ne[r, j], nts[r, j]) == (other, e, tt)
        assert np.all(nbr[r, cnt[r]:] == -1) and np.all(ne[r, cnt[r]:] == -1)


def test_self_loop_listed_twice_and_strict_past():
    src = np.array([0, 1, 1]); dst = np.array([1, 1, 2]); ts = np.array([1.0, 2.0, 3.0])
    for sample in (lambda *q: O.sample_recent(src, dst, ts, *q),
                   lambda *q: O.sample_recent_indexed(O.build_adjacency(src, dst, ts, 3), *q)):
        nbr, ne, nts, cnt = sample(np.array([1, 1, 0, 2]), np.array([3.0, 2.0, 1.0, 9.0]), 4)
        assert cnt.tolist() == [3, 1, 0, 1]
        assert ne[0, :3].tolist() == [1, 1, 0] and nbr[0, :3].tolist() == [1, 1, 0]
        assert ne[1, 0] == 0 and nts[1, 0] == 1.0                  # the event at t=2 is not < 2
        assert nbr[3, 0] == 1 and ne[3, 0] == 2


def test_invariants_on_c0():
    import synth
    g = synth.gen_graph("C0")
    adj = O.build_adjacency(g["src"], g["dst"], g["ts"], 1000)
    indptr, other, eid, tt = adj
    assert indptr[-1] == 2 * len(g["src"])
    # every event appears exactly twice; per-node lists ascend in (time, id)
    assert np.array_equal(np.sort(eid), np.repeat(np.arange(len(g["src"])), 2))
    for v in range(0, 1000, 37):
        seg = slice(indptr[v], indptr[v + 1])
        key = list(zip(tt[seg], eid[seg]))
        assert key == sorted(key)
    lo, hi = 5000, 5200
    qn = np.concatenate([g["src"][lo:hi], g["dst"][lo:hi]]); qt = np.concatenate([g["ts"][lo:hi]] * 2)
    nbr, ne, nts, cnt = O.sample_recent(g["src"], g["dst"], g["ts"], qn, qt, 10)
    for a, b in zip((nbr, ne, nts, cnt), O.sample_recent_indexed(adj, qn, qt, 10)):
        assert np.array_equal(a, b)
    m = np.arange(10)[None] < cnt[:, None]
    assert np.all(nts[m] < np.broadcast_to(qt[:, None], nts.shape)[m])
    assert np.all(np.diff(nts, axis=1)[m[:, 1:]] <= 0)                    # most recent first
    assert np.all(g["ts"][ne[m]] == nts[m])
    # the other endpoint of the listed event is the listed neighbour
    other_end = np.where(g["src"][ne[m]] == np.broadcast_to(qn[:, None], ne.shape)[m], g["dst"][ne[m]], g["src"][ne[m]])
    assert np.array_equal(other_end, nbr[m])
