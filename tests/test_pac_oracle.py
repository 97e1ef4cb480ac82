"""Pins of the epoch-machinery oracle (oracle/pac_oracle.py): Sec. II-C "Distributed Parallel
Training", Alg. 2."""
import numpy as np
import pytest

import tig_synth as S
from oracle import pac_oracle as E
from oracle import sep_oracle as P
from oracle import tig_oracle as O


def test_subgraph_by_hand():
    # 6 nodes, 3 parts; node 0 is shared (parts 0 and 2), node 5 never occurs
    node_parts = [0b101, 0b001, 0b010, 0b010, 0b100, 0]
    src = np.array([0, 1, 2, 0, 4, 1, 3])
    dst = np.array([1, 2, 3, 4, 0, 0, 0])
    # part 1 alone: nodes {0 (shared), 2, 3}: events (2,3), (3,0)
    eids, local, n = E.subgraph(src, dst, node_parts, 3, 0b010)
    assert eids.tolist() == [2, 6] and n == 3 and local.tolist() == [0, -1, 1, 2, -1, -1]
    # parts 0 and 2 combined: nodes {0, 1, 4}: the edge (1,0)/(0,1) inside part 0, (0,4)/(4,0) inside part 2
    eids, local, n = E.subgraph(src, dst, node_parts, 3, 0b101)
    assert eids.tolist() == [0, 3, 4, 5] and local.tolist() == [0, 1, -1, -1, 2, -1]
    # all parts: everything whose endpoints occur at all
    assert E.subgraph(src, dst, node_parts, 3, 0b111)[0].tolist() == list(range(7))


def test_combine_restores_edges_between_joined_parts():
    w = S.WORKLOADS["c1_tiny"]
    g = S.make_graph(w)
    r = P.partition(g.src, g.dst, g.ts, g.num_nodes, 8, beta=1e-5, k_frac=0.02, lam=1.0, eps=1e-3)
    masks = np.array([sum(1 << p for p in a) for a in r["A"]], dtype=np.uint64)
    order = np.random.default_rng(3).permutation(8)
    groups = E.combine(order, 4)
    assert sorted(groups) == sorted(sum(1 << int(p) for p in order[2 * i:2 * i + 2]) for i in range(4))
    assert sum(groups) == 0xFF and all(bin(m).count("1") == 2 for m in groups)
    for gm in groups:
        a, b = [p for p in range(8) if gm >> p & 1]
        ea = set(E.subgraph(g.src, g.dst, masks, 8, 1 << a)[0].tolist())
        eb = set(E.subgraph(g.src, g.dst, masks, 8, 1 << b)[0].tolist())
        eab = set(E.subgraph(g.src, g.dst, masks, 8, gm)[0].tolist())
        assert ea | eb <= eab                      # E_a u E_b u DE_ab
        ma, mb = E.members(masks, 8, 1 << a), E.members(masks, 8, 1 << b)
        extra = eab - ea - eb
        for e in extra:                            # the restored edges run between the two parts
            i, j = g.src[e], g.dst[e]
            assert (ma[i] and mb[j]) or (mb[i] and ma[j])
    # every event the stream kept lies in the sub-graph of its part
    for p in range(8):
        ep = set(E.subgraph(g.src, g.dst, masks, 8, 1 << p)[0].tolist())
        assert set(np.flatnonzero(r["edge_part"] == p).tolist()) <= ep


def _part(w, g, W, eids, local, n_local, batch):
    return {"num_nodes": n_local, "mem_dim": w.mem_dim, "src": local[g.src[eids]], "dst": local[g.dst[eids]],
            "ts": g.ts[eids], "edge_feat": g.edge_feat[eids], "W": W, "batch": batch, "neg": None}


def test_epoch_loop_resets_backs_up_and_restores():
    w = S.WORKLOADS["c1_tiny"].scaled(num_events=700)
    g = S.make_graph(w)
    W = S.make_weights(w)
    node_parts = np.full(g.num_nodes, 1, dtype=np.uint64)
    parts = []
    for lo, hi in ((0, 250), (250, 700)):      # 3 batches of 100 (last 50) and 5 (last 50)
        eids = np.arange(lo, hi)
        local = np.arange(g.num_nodes, dtype=np.int32)
        parts.append(_part(w, g, W, eids, local, g.num_nodes, 100))
    final, trace, steps = E.epoch(parts, w.num_neighbors, w.num_heads)
    assert steps == 5
    assert [(i, rs, bk) for _, i, rs, bk in trace[0]] == [(0, True, False), (1, False, False), (2, False, True),
                                                         (0, True, False), (1, False, False)]
    assert [(i, rs, bk) for _, i, rs, bk in trace[1]] == [(0, True, False), (1, False, False), (2, False, False),
                                                         (3, False, False), (4, False, True)]
    # the restored memory is the memory at the end of the partition's last COMPLETE data cycle
    for k, p in enumerate(parts):
        st = O.OracleState.zeros(p["num_nodes"], p["mem_dim"])
        for first in range(0, len(p["src"]), 100):
            O.step(st, p["src"], p["dst"], p["ts"], p["edge_feat"], W, first, min(100, len(p["src"]) - first), None,
                   w.num_neighbors, w.num_heads)
        assert np.array_equal(final[k].mem, st.mem) and np.array_equal(final[k].last_update, st.last_update)


def test_sync_shared_rules_by_hand():
    def states():
        a, b, c = (O.OracleState.zeros(4, 2) for _ in range(3))
        a.mem[1], a.last_update[1] = [1, 2], 5.0
        b.mem[0], b.last_update[0] = [3, 5], 9.0
        c.mem[2], c.last_update[2] = [8, 8], 9.0
        a.mem[3], b.mem[3], c.mem[3] = [7, 7], [7, 7], [7, 7]
        return [a, b, c]
    ids = [[1], [0], [2]]                      # one shared node: row 1 / 0 / 2 in the three partitions
    st = states()
    E.sync_shared(st, ids, "latest")           # times 5, 9, 9: the lowest partition with the largest time wins
    for s, r in zip(st, (1, 0, 2)):
        assert s.mem[r].tolist() == [3, 5] and s.last_update[r] == 9.0
        assert s.mem[3].tolist() == [7, 7]     # other rows untouched
    st = states()
    E.sync_shared(st, ids, "mean")
    for s, r in zip(st, (1, 0, 2)):
        assert s.mem[r].tolist() == [4, 5] and s.last_update[r] == 9.0
