"""Pins for the oracle's most-recent-neighbour sampler: a brute-force scan of the raw event list
(Sec. 2.1 "most recent neighbors"), plus the strict-past invariant."""
import numpy as np
import pytest

from oracle import tgnn_oracle as O


def brute_force(src, dst, ts, node, t, k):
    """Scan all events; keep those touching `node` with time < t; order by (time, id); take last k."""
    cand = []
    for e in range(len(src)):
        if ts[e] < t:
            if src[e] == node:
                cand.append((ts[e], e, dst[e]))
            if dst[e] == node:
                cand.append((ts[e], e, src[e]))
    cand.sort(key=lambda c: (c[0], c[1]))
    return cand[::-1][:k]


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_sampler_vs_bruteforce_with_ties(seed):
    rng = np.random.default_rng(seed)
    n, E, k = 30, 400, 5
    src = rng.integers(0, n - 3, E); dst = rng.integers(0, n - 3, E)      # nodes n-3.. have no events
    ts = np.sort(rng.integers(0, 60, E)).astype(np.float64)               # many equal timestamps
    adj = O.build_adjacency(src, dst, ts, n)
    qn = rng.integers(0, n, 300); qt = rng.integers(-1, 62, 300).astype(np.float64)
    nbr, ne, nts, cnt = O.sample_recent(adj, qn, qt, k)
    for r in range(len(qn)):
        ref = brute_force(src, dst, ts, qn[r], qt[r], k)
        assert cnt[r] == len(ref)
        for j, (tt, e, other) in enumerate(ref):
            assert (nbr[r, j], ne[r, j], nts[r, j]) == (other, e, tt)
        assert np.all(nbr[r, cnt[r]:] == -1) and np.all(ne[r, cnt[r]:] == -1)


def test_self_loop_listed_twice_and_strict_past():
    src = np.array([0, 1, 1]); dst = np.array([1, 1, 2]); ts = np.array([1.0, 2.0, 3.0])
    adj = O.build_adjacency(src, dst, ts, 3)
    nbr, ne, nts, cnt = O.sample_recent(adj, np.array([1, 1, 0, 2]), np.array([3.0, 2.0, 1.0, 9.0]), 4)
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
    nbr, ne, nts, cnt = O.sample_recent(adj, qn, qt, 10)
    m = np.arange(10)[None] < cnt[:, None]
    assert np.all(nts[m] < np.broadcast_to(qt[:, None], nts.shape)[m])
    assert np.all(np.diff(nts, axis=1)[m[:, 1:]] <= 0)                    # most recent first
    assert np.all(g["ts"][ne[m]] == nts[m])
