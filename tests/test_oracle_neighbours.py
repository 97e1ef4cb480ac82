"""Pins for the most-recent-K temporal neighbour lookup of the oracle."""
import numpy as np
import pytest

import tig_synth as S
from oracle import tig_oracle as O


def _independent(src, dst, ts, u, t, K):
    """A separate statement of the definition with Python's sorted()."""
    rows = [(float(ts[e]), e, int(dst[e]) if src[e] == u else int(src[e]))
            for e in range(len(src)) if (src[e] == u or dst[e] == u) and ts[e] < t]
    rows = sorted(rows, reverse=True)[:K]
    return rows


def _check_query(src, dst, ts, u, t, K, got):
    nb_node, nb_eid, nb_ts, cnt = got
    rows = _independent(src, dst, ts, u, t, K)
    assert cnt == len(rows)
    for k, (tt, e, v) in enumerate(rows):
        assert (nb_eid[k], nb_node[k], nb_ts[k]) == (e, v, tt)
    assert np.all(nb_eid[cnt:] == -1) and np.all(nb_node[cnt:] == -1) and np.all(nb_ts[cnt:] == 0.0)


def test_bruteforce_matches_independent_sort_random():
    rng = np.random.default_rng(0)
    E, N, K = 600, 15, 4
    src = rng.integers(0, N, size=E).astype(np.int32)
    dst = ((src + rng.integers(1, N, size=E)) % N).astype(np.int32)
    ts = np.sort(rng.integers(0, 80, size=E)).astype(np.float64)   # many ties
    for _ in range(200):
        u = int(rng.integers(0, N))
        t = float(rng.integers(0, 82)) + float(rng.choice([0.0, 0.5]))
        _check_query(src, dst, ts, u, t, K, O.neighbours_bruteforce(src, dst, ts, u, t, K))


def test_hand_cases():
    # node 0 meets 1, 2, 1, 3 at times 1, 2, 2, 5; node 4 never appears
    src = np.array([0, 2, 0, 3, 1], dtype=np.int32)
    dst = np.array([1, 0, 1, 0, 2], dtype=np.int32)
    ts = np.array([1.0, 2.0, 2.0, 5.0, 5.0])
    nb = lambda u, t, K: O.neighbours_bruteforce(src, dst, ts, u, t, K)
    # strictly earlier: the query's own time is excluded
    node, eid, tt, cnt = nb(0, 2.0, 3)
    assert cnt == 1 and eid.tolist() == [0, -1, -1] and node.tolist() == [1, -1, -1]
    # ties ordered by event id, most recent first; duplicate pair (0,1) kept twice
    node, eid, tt, cnt = nb(0, 5.0, 3)
    assert cnt == 3 and eid.tolist() == [2, 1, 0] and node.tolist() == [1, 2, 1]
    assert tt.tolist() == [2.0, 2.0, 1.0]
    # exactly K and K + 1 earlier events
    assert nb(0, 6.0, 4)[1].tolist() == [3, 2, 1, 0]
    assert nb(0, 6.0, 3)[1].tolist() == [3, 2, 1]
    # query at the first timestamp, and a node without events
    assert nb(0, 1.0, 2)[3] == 0
    assert nb(4, 100.0, 2)[3] == 0
    # all-equal timestamps: nothing is strictly earlier
    same = np.full(5, 3.0)
    assert O.neighbours_bruteforce(src, dst, same, 0, 3.0, 2)[3] == 0


def test_index_matches_bruteforce_on_small_workloads():
    for w in (S.WORKLOADS["c1_tiny"],
              S.WORKLOADS["c2_bipartite_medium"].scaled(num_events=20000),
              S.WORKLOADS["c3_bipartite_dense"].scaled(num_events=20000)):
        g = S.make_graph(w, with_features=False)
        ix = O.NeighbourIndex(g.num_nodes, g.src, g.dst, g.ts)
        rng = np.random.default_rng(w.index)
        ev = rng.integers(0, g.num_events, size=300)
        nodes = np.concatenate([g.src[ev], g.dst[ev], rng.integers(0, g.num_nodes, size=300)])
        times = np.concatenate([g.ts[ev], g.ts[ev], g.ts[ev]])
        K = w.num_neighbors
        a = ix.query(nodes.astype(np.int32), times, K)
        b = O.neighbours_bruteforce_batch(g.src, g.dst, g.ts, nodes, times, K)
        for x, y in zip(a, b):
            np.testing.assert_array_equal(x, y)
        # invariants: no future leakage; slots strictly decreasing in (time, event id)
        nb_node, nb_eid, nb_ts, cnt = a
        for q in range(len(nodes)):
            c = cnt[q]
            assert np.all(nb_ts[q, :c] < times[q])
            keys = list(zip(nb_ts[q, :c], nb_eid[q, :c]))
            assert keys == sorted(keys, reverse=True) and len(set(keys)) == c
            for k in range(c):
                e = nb_eid[q, k]
                assert {int(g.src[e]), int(g.dst[e])} == {int(nodes[q]), int(nb_node[q, k])}
        assert (g.ts == np.floor(g.ts)).all() == w.integer_seconds


def test_index_rejects_bad_graphs():
    src = np.array([0, 1], dtype=np.int32)
    dst = np.array([1, 2], dtype=np.int32)
    with pytest.raises(ValueError):
        O.NeighbourIndex(3, src, dst, np.array([2.0, 1.0]))      # unsorted
    with pytest.raises(ValueError):
        O.NeighbourIndex(2, src, dst, np.array([1.0, 2.0]))      # id out of range
