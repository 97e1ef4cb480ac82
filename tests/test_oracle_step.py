"""Pins for the whole oracle step: data-flow order and layouts (through selector weights whose
result can be written down by hand), and the invariants the method guarantees."""
import math

import numpy as np
import pytest

import tig_synth as S
from oracle import tig_oracle as O

M, T, F, E = 2, 2, 2, 2
D_MSG, D_A, D_KV = 2 * M + T + F, M + T, M + F + T
BIG = 100.0


def _zero_weights():
    W = {k: np.zeros(s, dtype=np.float32) for k, s in S.weight_shapes(M, T, F, E).items()}
    W["time_w"][:] = [0.5, 0.01]
    W["time_b"][:] = [0.3, -1.1]
    return W


def _tiny_graph():
    #          e: 0  1  2  3   4  5
    src = np.array([0, 3, 1, 2, 0, 2], dtype=np.int32)
    dst = np.array([1, 0, 2, 3, 1, 0], dtype=np.int32)
    ts = np.array([1.0, 2.0, 3.0, 4.0, 10.0, 12.0])
    rng = np.random.default_rng(11)
    feat = rng.normal(size=(6, F)).astype(np.float32)
    return src, dst, ts, feat


def _state():
    rng = np.random.default_rng(12)
    return O.OracleState(rng.uniform(-1, 1, size=(4, M)).astype(np.float32),
                         np.array([2.0, 3.0, 4.0, 4.0]))


def _phi(W, x):
    return np.cos(W["time_w"].astype(np.float64) * x + W["time_b"].astype(np.float64)).astype(np.float32)


@pytest.mark.parametrize("sel", range(D_MSG))
def test_message_layout_and_update(sel):
    """Batch = events 4 (0->1, t=10) and 5 (2->0, t=12).  With the update gate shut (z = 0) and
    W_in a selector, the new memory entry 0 is tanh(message[sel]), so the message layout
    [own | other | Phi(t - last_update[own]) | edge feature], the use of batch-start memory
    for BOTH endpoints, and the winner choice are all visible."""
    src, dst, ts, feat = _tiny_graph()
    W = _zero_weights()
    W["b_i"][M:2 * M] = -400.0
    W["W_i"][2 * M, sel] = 1.0
    st = _state()
    mem0, lu0 = st.mem.copy(), st.last_update.copy()
    out = O.step(st, src, dst, ts, feat, W, first_eid=4, count=2, neg_dst=None, K=2, H=2)
    msg = {
        0: np.concatenate([mem0[0], mem0[2], _phi(W, 12.0 - lu0[0]), feat[5]]),   # last: event 5, as dst
        1: np.concatenate([mem0[1], mem0[0], _phi(W, 10.0 - lu0[1]), feat[4]]),   # event 4, as dst
        2: np.concatenate([mem0[2], mem0[0], _phi(W, 12.0 - lu0[2]), feat[5]]),   # event 5, as src
    }
    for u, m in msg.items():
        assert st.mem[u, 0] == np.float32(math.tanh(float(m[sel])))
        assert st.mem[u, 1] == 0.0                      # tanh(0): row 1 of W_in is zero
    assert st.last_update.tolist() == [12.0, 10.0, 12.0, 4.0]
    # node 3 is not in the batch: untouched
    assert np.array_equal(st.mem[3], mem0[3])
    # entries are (2b + role); event 4's source (node 0) loses to event 5's destination
    assert out["is_winner"].tolist() == [0, 1, 1, 1]


@pytest.mark.parametrize("sel", range(D_KV))
def test_key_value_layout_and_post_update_memory(sel):
    """Query (node 1, t = 3.0) has exactly one earlier event: event 0 with node 0.  With one
    neighbour the attention weight is 1 and attn = W_O (W_V kv + b_V) + b_O.  Selector weights
    carry kv[sel] to emb[.., 0].  Node 0's memory is rewritten by this very batch (it is the
    destination of event 1... and here of event 2's batch), so kv[0:M] must be the UPDATED row."""
    src, dst, ts, feat = _tiny_graph()
    W = _zero_weights()
    # GRU that maps every touched node's memory to tanh of its own first message entry
    W["b_i"][M:2 * M] = -400.0
    W["W_i"][2 * M, 0] = 1.0
    W["W_i"][2 * M + 1, 1] = 1.0
    W["W_V"][0, sel] = 1.0
    W["W_O"][:] = np.eye(D_A)
    W["W_m1"][0, 0] = 1.0
    W["b_m1"][0] = BIG
    W["W_m2"][:] = np.eye(E)
    W["b_m2"][0] = -BIG
    st = _state()
    mem0 = st.mem.copy()
    # batch = events 1 (3->0, t=2) and 2 (1->2, t=3): queries are (3,2),(1,3),(0,2),(2,3)
    out = O.step(st, src, dst, ts, feat, W, first_eid=1, count=2, neg_dst=None, K=3, H=2)
    assert out["q_node"].tolist() == [3, 1, 0, 2]
    q = 1                                               # (node 1, t = 3.0)
    assert out["nbr_cnt"][q] == 1 and out["nbr_eid"][q, 0] == 0 and out["nbr_node"][q, 0] == 0
    new0 = np.tanh(mem0[0].astype(np.float64)).astype(np.float32)   # node 0 updated by event 1
    assert np.array_equal(st.mem[0], new0)
    kv = np.concatenate([new0, feat[0], _phi(W, 3.0 - 1.0)])
    np.testing.assert_allclose(out["emb"][q, 0], kv[sel], rtol=0, atol=2e-5)  # (x+100)-100 in fp64->fp32
    # query (node 3, t = 2.0): nothing strictly earlier -> attn = 0 -> emb = relu(b_m1) + b_m2 = 0
    assert out["nbr_cnt"][0] == 0
    np.testing.assert_allclose(out["emb"][0], [0.0, 0.0], atol=1e-6)


def test_query_vector_layout_and_scores():
    """Two neighbours; W_Q and W_K select single entries so that the score is
    q_in[a] * kv[b] / sqrt(d_h).  q_in = [updated memory of the query node | Phi(0)]."""
    src, dst, ts, feat = _tiny_graph()
    for a in range(D_A):
        W = _zero_weights()
        W["W_Q"][0, a] = 1.0
        W["W_K"][0, M] = 4.0                 # first edge-feature entry of the key row
        W["W_V"][0, M + 1] = 1.0             # second edge-feature entry as the value
        W["W_O"][:] = np.eye(D_A)
        W["W_m1"][0, 0] = 1.0
        W["b_m1"][0] = BIG
        W["W_m2"][:] = np.eye(E)
        W["b_m2"][0] = -BIG
        st = _state()
        mem0 = st.mem.copy()
        # batch = event 5 alone (2->0, t=12); query (0, 12): history events 4, 1, 0 -> K=2: 4, 1
        out = O.step(st, src, dst, ts, feat, W, first_eid=5, count=1, neg_dst=None, K=2, H=1)
        q = 1
        assert out["nbr_eid"][q].tolist() == [4, 1]
        # all GRU parameters are zero here, so the update halves the row
        q_in = np.concatenate([(0.5 * mem0[0].astype(np.float64)).astype(np.float32), _phi(W, 0.0)])
        s = np.array([q_in[a] * 4.0 * feat[4, 0], q_in[a] * 4.0 * feat[1, 0]], dtype=np.float64) / math.sqrt(D_A)
        p = np.exp(s - s.max())
        p /= p.sum()
        want = p[0] * feat[4, 1] + p[1] * feat[1, 1]
        np.testing.assert_allclose(out["emb"][q, 0], want, rtol=0, atol=2e-5)


def test_decoder_pairs_and_row_order():
    w = S.WORKLOADS["c1_tiny"].scaled(num_events=400)
    g = S.make_graph(w)
    W = S.make_weights(w)
    Ed = w.emb_dim
    W["W_d1"][:] = 0
    W["W_d1"][0, 0] = 1.0            # first entry of the first embedding of the pair
    W["W_d1"][1, Ed + 1] = 1.0       # second entry of the second embedding
    W["b_d1"][:] = 0
    W["b_d1"][:2] = BIG
    W["w_d2"][:] = 0
    W["w_d2"][:2] = 1.0
    W["b_d2"][0] = -2 * BIG
    st = O.OracleState.zeros(g.num_nodes, w.mem_dim)
    first, count = 200, 50
    neg = S.make_negatives(w, g, first, count)
    out = O.step(st, g.src, g.dst, g.ts, g.edge_feat, W, first, count, neg, w.num_neighbors, w.num_heads)
    emb = out["emb"].astype(np.float64)
    assert out["q_node"].tolist() == g.src[first:first + count].tolist() + \
        g.dst[first:first + count].tolist() + neg.tolist()
    np.testing.assert_allclose(out["score_pos"], emb[:count, 0] + emb[count:2 * count, 1], atol=2e-5)
    np.testing.assert_allclose(out["score_neg"], emb[:count, 0] + emb[2 * count:, 1], atol=2e-5)


def test_step_invariants_c1():
    w = S.WORKLOADS["c1_tiny"]
    g = S.make_graph(w)
    W = S.make_weights(w)
    st = O.OracleState.zeros(g.num_nodes, w.mem_dim)
    ix = O.NeighbourIndex(g.num_nodes, g.src, g.dst, g.ts)
    for first, count in list(S.batches(g.num_events, w.batch_size))[:6]:
        before = st.copy()
        neg = S.make_negatives(w, g, first, count)
        out = O.step(st, g.src, g.dst, g.ts, g.edge_feat, W, first, count, neg, w.num_neighbors,
                     w.num_heads, index=ix)
        touched = np.zeros(g.num_nodes, dtype=bool)
        touched[g.src[first:first + count]] = True
        touched[g.dst[first:first + count]] = True
        # memory and last_update are bit-identical for nodes without an event in the batch
        assert np.array_equal(st.mem[~touched], before.mem[~touched])
        assert np.array_equal(st.last_update[~touched], before.last_update[~touched])
        # every touched node now carries the time of its last event in the batch
        for u in np.flatnonzero(touched):
            bs = np.flatnonzero((g.src[first:first + count] == u) | (g.dst[first:first + count] == u))
            assert st.last_update[u] == g.ts[first + bs.max()]
        # one winner per distinct node
        assert out["is_winner"].sum() == touched.sum()
        # no future leakage
        valid = out["nbr_eid"] >= 0
        assert np.all(out["nbr_ts"][valid] < np.repeat(out["q_time"], w.num_neighbors).reshape(valid.shape)[valid])
        assert np.all(np.isfinite(out["emb"])) and np.all(np.isfinite(out["score_pos"]))


def test_indexed_and_bruteforce_steps_agree():
    w = S.WORKLOADS["c1_tiny"].scaled(num_events=1500)
    g = S.make_graph(w)
    W = S.make_weights(w)
    a = O.OracleState.zeros(g.num_nodes, w.mem_dim)
    b = O.OracleState.zeros(g.num_nodes, w.mem_dim)
    ix = O.NeighbourIndex(g.num_nodes, g.src, g.dst, g.ts)
    for first, count in S.batches(g.num_events, 300):
        neg = S.make_negatives(w, g, first, count)
        oa = O.step(a, g.src, g.dst, g.ts, g.edge_feat, W, first, count, neg, 10, 2, index=None)
        ob = O.step(b, g.src, g.dst, g.ts, g.edge_feat, W, first, count, neg, 10, 2, index=ix)
        for k in ("emb", "score_pos", "score_neg", "nbr_node", "nbr_eid", "nbr_ts", "nbr_cnt", "is_winner"):
            assert np.array_equal(oa[k], ob[k]), k
    assert np.array_equal(a.mem, b.mem) and np.array_equal(a.last_update, b.last_update)


def test_disjoint_batch_is_order_independent():
    """Events of one batch that touch pairwise-disjoint nodes and share a timestamp can be
    listed in any order: the state after the step is the same."""
    rng = np.random.default_rng(13)
    w = S.WORKLOADS["c1_tiny"]
    W = S.make_weights(w)
    N, B = 40, 12
    hist_src = rng.integers(0, N, size=60).astype(np.int32)
    hist_dst = ((hist_src + rng.integers(1, N, size=60)) % N).astype(np.int32)
    hist_ts = np.sort(rng.uniform(0, 50, size=60))
    nodes = rng.permutation(N)[:2 * B].astype(np.int32)
    bs, bd = nodes[:B], nodes[B:]
    feat_h = rng.normal(size=(60, w.feat_dim)).astype(np.float32)
    feat_b = rng.normal(size=(B, w.feat_dim)).astype(np.float32)
    mem = rng.uniform(-1, 1, size=(N, w.mem_dim)).astype(np.float32)
    lu = rng.uniform(0, 50, size=N)
    results = []
    for perm in (np.arange(B), rng.permutation(B)):
        src = np.concatenate([hist_src, bs[perm]])
        dst = np.concatenate([hist_dst, bd[perm]])
        ts = np.concatenate([hist_ts, np.full(B, 60.0)])
        feat = np.concatenate([feat_h, feat_b[perm]])
        st = O.OracleState(mem.copy(), lu.copy())
        out = O.step(st, src, dst, ts, feat, W, 60, B, None, w.num_neighbors, w.num_heads)
        inv = np.argsort(perm)
        results.append((st.mem.copy(), st.last_update.copy(), out["score_pos"][inv]))
    assert np.array_equal(results[0][0], results[1][0])
    assert np.array_equal(results[0][1], results[1][1])
    assert np.array_equal(results[0][2], results[1][2])


def test_reset_state_is_zero():
    st = O.OracleState.zeros(5, 3)
    assert st.mem.dtype == np.float32 and st.last_update.dtype == np.float64
    assert not st.mem.any() and not st.last_update.any()


# ------------------------------------------------------------------------ deferred order


def _c1_setup():
    w = S.WORKLOADS["c1_tiny"].scaled(num_events=1200)
    g = S.make_graph(w)
    W = S.make_weights(w)
    return w, g, W


def test_deferred_memory_equals_update_first_of_the_previous_batch():
    """After deferred steps over batches b1, b2 the memory is what the update-first step over b1
    leaves (b2's messages are still waiting), and after b3 what update-first over b1, b2 leaves;
    the first deferred step after a reset applies nothing."""
    w, g, W = _c1_setup()
    bs = [(200, 100), (300, 100), (400, 150)]
    a = O.OracleState(*S.make_warm_state(w, g, 200))
    b = a.copy()
    mem_start, lu_start = a.mem.copy(), a.last_update.copy()
    kw = dict(K=w.num_neighbors, H=w.num_heads)
    O.step(a, g.src, g.dst, g.ts, g.edge_feat, W, *bs[0], None, deferred=True, **kw)
    assert np.array_equal(a.mem, mem_start) and np.array_equal(a.last_update, lu_start)
    assert len(a.pending) > 0
    for k in (1, 2):
        O.step(a, g.src, g.dst, g.ts, g.edge_feat, W, *bs[k], None, deferred=True, **kw)
        O.step(b, g.src, g.dst, g.ts, g.edge_feat, W, *bs[k - 1], None, **kw)
        assert np.array_equal(a.mem, b.mem) and np.array_equal(a.last_update, b.last_update)
    # what is kept are the winners of the last batch: one per distinct node, its last occurrence
    nodes = {u for u, _, _, _ in a.pending}
    first, count = bs[2]
    assert nodes == set(g.src[first:first + count]) | set(g.dst[first:first + count])
    for u, other, eid, t in a.pending:
        later = [e for e in range(eid + 1, first + count) if g.src[e] == u or g.dst[e] == u]
        assert not later and t == g.ts[eid] and {u, other} == {int(g.src[eid]), int(g.dst[eid])}


def test_deferred_embeds_from_the_memory_the_applied_messages_leave():
    """The deferred step over b2 embeds from the memory that the update-first step over b1 leaves.
    An update-first step over b2 on that memory, with a GRU whose update gate is stuck at 1 (so
    its own update keeps every row), produces exactly the embedding function on that memory."""
    w, g, W = _c1_setup()
    b1, b2 = (200, 100), (300, 100)
    neg = S.make_negatives(w, g, *b2)
    kw = dict(K=w.num_neighbors, H=w.num_heads)
    a = O.OracleState(*S.make_warm_state(w, g, 200))
    ref = a.copy()
    O.step(a, g.src, g.dst, g.ts, g.edge_feat, W, *b1, None, deferred=True, **kw)
    out_a = O.step(a, g.src, g.dst, g.ts, g.edge_feat, W, *b2, neg, deferred=True, **kw)
    O.step(ref, g.src, g.dst, g.ts, g.edge_feat, W, *b1, None, **kw)
    keep = {k: v.copy() for k, v in W.items()}
    keep["b_i"][w.mem_dim:2 * w.mem_dim] = 400.0        # z = sigmoid(+large) = 1  ->  h' = h
    mem_before = ref.mem.copy()
    out_r = O.step(ref, g.src, g.dst, g.ts, g.edge_feat, keep, *b2, neg, **kw)
    assert np.array_equal(ref.mem, mem_before)
    for name in ("emb", "score_pos", "score_neg", "nbr_node", "nbr_eid", "nbr_cnt", "is_winner"):
        assert np.array_equal(out_a[name], out_r[name]), name


def test_dropping_what_is_kept():
    w, g, W = _c1_setup()
    kw = dict(K=w.num_neighbors, H=w.num_heads)
    a = O.OracleState(*S.make_warm_state(w, g, 200))
    O.step(a, g.src, g.dst, g.ts, g.edge_feat, W, 200, 100, None, deferred=True, **kw)
    a.drop_pending()
    before = a.mem.copy()
    O.step(a, g.src, g.dst, g.ts, g.edge_feat, W, 300, 100, None, deferred=True, **kw)
    assert np.array_equal(a.mem, before)
