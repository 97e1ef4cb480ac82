"""Pins for the two-layer attention embedding of the oracle (Sec. II-C embedding module: the sum runs
over the k-hop temporal neighbourhood neighbor_i^k([0, t]); k = 2 as two stacked attention layers).
None retypes the recursion: a pass-through second layer, a second layer that averages its
neighbour rows checked against the pinned ONE-layer step (which embeds any node at an event's
time when it is handed over as that event's negative), a hand-built chain graph, truncation of
the future."""
import numpy as np
import pytest

import tig_synth as S
from oracle import modules_oracle as G
from oracle import tig_oracle as O

C = 10.0  # offset that carries a row through the ReLU of a merge MLP unchanged


def _c1():
    w = S.WORKLOADS["c1_tiny"]
    g, W = S.make_graph(w), S.make_weights(w)
    ix = O.NeighbourIndex(g.num_nodes, g.src, g.dst, g.ts)
    st = O.OracleState(*S.make_warm_state(w, g, 4000))
    return w, g, W, ix, st


def _copy(st):
    return O.OracleState(st.mem.copy(), st.last_update.copy())


def _zero_layer2(w):
    return {k: np.zeros_like(v) for k, v in S.make_layer2_weights(w).items()}


def _merge_selects(L2, E, first_col):
    """merge MLP of the second layer = the E columns of [attn | h_self] starting at first_col."""
    L2["W_m1"][np.arange(E), first_col + np.arange(E)] = 1.0
    L2["b_m1"][:] = C
    L2["W_m2"][np.arange(E), np.arange(E)] = 1.0
    L2["b_m2"][:] = -C


def test_layer2_weight_shapes():
    w = S.WORKLOADS["c2_bipartite_medium"]   # E != M
    L2 = S.make_layer2_weights(w)
    E, T, F = w.emb_dim, w.time_dim, w.feat_dim
    assert L2["W_Q"].shape == (E + T, E + T) and L2["W_K"].shape == (E + T, E + F + T)
    assert L2["W_V"].shape == (E + T, E + F + T) and L2["W_O"].shape == (E + T, E + T)
    assert L2["W_m1"].shape == (E, 2 * E + T) and L2["W_m2"].shape == (E, E)


def test_pass_through_second_layer_returns_the_first_layers_rows():
    w, g, W, ix, st = _c1()
    E = w.emb_dim
    L2 = _zero_layer2(w)                         # attention of layer 2 contributes the zero vector
    _merge_selects(L2, E, E + w.time_dim)        # h_self follows the [E + T] attention columns
    first, count = 4000, 60
    neg = S.make_negatives(w, g, first, count)
    one = G.step(_copy(st), g.src, g.dst, g.ts, g.edge_feat, W, first, count, neg, w.num_neighbors, w.num_heads,
                 G.Modules(), index=ix)
    two = G.step(_copy(st), g.src, g.dst, g.ts, g.edge_feat, W, first, count, neg, w.num_neighbors, w.num_heads,
                 G.Modules(layers=2, layer2=L2), index=ix)
    np.testing.assert_allclose(two["emb"], one["emb"], rtol=0, atol=2e-6)
    for k in ("nbr_node", "nbr_eid", "nbr_ts", "nbr_cnt", "is_winner"):
        np.testing.assert_array_equal(two[k], one[k])
    np.testing.assert_allclose(two["score_pos"], one["score_pos"], rtol=0, atol=1e-5)


def test_averaging_second_layer_gives_the_mean_of_the_neighbours_one_layer_rows():
    """Zero query projection => uniform attention; the value projection keeps the neighbour's row;
    so layer 2 returns mean_k h1_{v_k}(t).  Each h1_{v_k}(t) is taken from the pinned one-layer step
    tig_oracle.step, which embeds v_k at time t_b when v_k is event b's negative."""
    w, g, W, ix, st = _c1()
    E, K = w.emb_dim, w.num_neighbors
    L2 = _zero_layer2(w)
    L2["W_V"][np.arange(E), np.arange(E)] = 1.0
    L2["W_O"][np.arange(E + w.time_dim), np.arange(E + w.time_dim)] = 1.0
    _merge_selects(L2, E, 0)
    first, count = 4000, 40
    two = G.step(_copy(st), g.src, g.dst, g.ts, g.edge_feat, W, first, count, None, K, w.num_heads,
                 G.Modules(layers=2, layer2=L2), index=ix)
    for role in (0, 1):
        rows = np.zeros((count, K, E))
        for k in range(K):
            col = two["nbr_node"][role * count:(role + 1) * count, k]
            neg = np.where(col >= 0, col, 0).astype(np.int32)
            one = O.step(_copy(st), g.src, g.dst, g.ts, g.edge_feat, W, first, count, neg, K, w.num_heads, ix)
            rows[:, k] = one["emb"][2 * count:]
        for b in range(count):
            c = int(two["nbr_cnt"][role * count + b])
            want = rows[b, :c].mean(axis=0) if c else np.zeros(E)
            np.testing.assert_allclose(two["emb"][role * count + b], want, rtol=0, atol=3e-6)
    assert int(two["nbr_cnt"].max()) == K and int((two["nbr_cnt"] > 1).sum()) > 10  # the mean is over several rows


def _chain():
    # node:  0 -- 1 -- 2      1 -- 4 (later than 0--1)      5 -- 2 (three hops from 0)
    src = np.array([1, 5, 0, 1, 0], dtype=np.int32)
    dst = np.array([2, 2, 1, 4, 3], dtype=np.int32)
    ts = np.array([1.0, 1.5, 2.0, 2.5, 3.0])
    return src, dst, ts


@pytest.mark.parametrize("layers", [1, 2])
def test_chain_graph_second_hop_is_seen_by_two_layers_only_and_at_the_query_time(layers):
    """Query (0, t = 3): hop 1 is node 1 (event at 2.0).  Node 1's row AT t = 3 sees node 2 (1.0) and
    node 4 (2.5 -- later than the event that links 0 and 1, earlier than the query).  Node 5 is three
    hops away."""
    w = S.WORKLOADS["c1_tiny"]
    W, L2 = S.make_weights(w), S.make_layer2_weights(w)
    src, dst, ts = _chain()
    feat = np.random.default_rng(5).normal(size=(5, w.feat_dim)).astype(np.float32)
    rng = np.random.default_rng(6)
    mem = rng.uniform(-1, 1, size=(6, w.mem_dim)).astype(np.float32)
    lu = np.zeros(6)
    mods = G.Modules(layers=layers, layer2=L2)
    lookup = lambda nodes, times: O.neighbours_bruteforce_batch(src, dst, ts, nodes, times, w.num_neighbors)

    def emb(m):
        return G.embed_layer(O.OracleState(m, lu.copy()), mods, W, feat, w.num_heads, lookup, layers, 0, 3.0)

    base = emb(mem)
    for node, seen_by in ((1, (1, 2)), (2, (2,)), (4, (2,)), (5, ()), (3, ())):
        m = mem.copy()
        m[node] += 1.0
        changed = not np.array_equal(emb(m), base)
        assert changed == (layers in seen_by), (node, layers)


def test_nothing_at_or_after_the_query_time_is_read_in_either_hop():
    w, g, W, ix, st = _c1()
    L2 = S.make_layer2_weights(w)
    mods = G.Modules(layers=2, layer2=L2)
    n = 1500
    src, dst, ts, feat = g.src[:n], g.dst[:n], g.ts[:n], g.edge_feat[:n]
    q = 900
    t = float(ts[q])
    cut = int(np.searchsorted(ts, t, side="left"))  # events [0, cut) are strictly earlier
    full = lambda nodes, times: O.neighbours_bruteforce_batch(src, dst, ts, nodes, times, w.num_neighbors)
    past = lambda nodes, times: O.neighbours_bruteforce_batch(src[:cut], dst[:cut], ts[:cut], nodes, times, w.num_neighbors)
    feat_past = feat.copy()
    feat_past[cut:] = 1e6   # would be visible at once
    for u in (int(src[q]), int(dst[q])):
        a = G.embed_layer(st, mods, W, feat, w.num_heads, full, 2, u, t)
        b = G.embed_layer(st, mods, W, feat_past, w.num_heads, past, 2, u, t)
        np.testing.assert_array_equal(a, b)
