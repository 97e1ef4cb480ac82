"""Pins for the oracle of the other instances of the general architecture (Sec. II-C: mean
aggregator, RNN update, identity / time-projection embedding; Sec. II-A: node features).  None of
them retypes the oracle's formula: reductions to the pinned headline oracle, values written out by
hand, closed forms, a float64 library cell."""
import math

import numpy as np
import pytest
import torch

import tig_synth as S
from oracle import modules_oracle as G
from oracle import tig_oracle as O

M, T, F = 2, 2, 2
D_MSG = 2 * M + T + F


def _graph():
    #          e: 0  1  2  3   4  5  6
    src = np.array([0, 3, 1, 2, 0, 2, 0], dtype=np.int32)
    dst = np.array([1, 0, 2, 3, 1, 0, 3], dtype=np.int32)
    ts = np.array([1.0, 2.0, 3.0, 4.0, 10.0, 12.0, 15.0])
    feat = np.random.default_rng(11).normal(size=(7, F)).astype(np.float32)
    return src, dst, ts, feat


def _state():
    rng = np.random.default_rng(12)
    return O.OracleState(rng.uniform(-1, 1, size=(4, M)).astype(np.float32), np.array([2.0, 3.0, 4.0, 4.0]))


def _weights(updater="gru", embedding="attention", E=2):
    W = {k: np.zeros(s, dtype=np.float32) for k, s in S.weight_shapes(M, T, F, E).items()}
    W["time_w"][:] = [0.5, 0.01]
    W["time_b"][:] = [0.3, -1.1]
    if updater == "rnn":
        W["W_i"], W["b_i"] = np.zeros((M, D_MSG), np.float32), np.zeros(M, np.float32)
        W["W_h"], W["b_h"] = np.zeros((M, M), np.float32), np.zeros(M, np.float32)
    if embedding == "time_projection":
        W["time_proj_w"] = np.array([0.25, -0.5], dtype=np.float32)
    return W


def _phi(W, x):
    return np.cos(W["time_w"].astype(np.float64) * x + W["time_b"].astype(np.float64)).astype(np.float32)


# ------------------------------------------------------------------ reduction to the headline oracle

@pytest.mark.parametrize("deferred", [False, True])
def test_headline_instance_is_the_pinned_step_bit_for_bit(deferred):
    w = S.WORKLOADS["c1_tiny"]
    g, W = S.make_graph(w), S.make_weights(w)
    a, b = O.OracleState.zeros(g.num_nodes, w.mem_dim), O.OracleState.zeros(g.num_nodes, w.mem_dim)
    ix = O.NeighbourIndex(g.num_nodes, g.src, g.dst, g.ts)
    for first in (0, 40, 80):
        neg = S.make_negatives(w, g, first, 40)
        ra = O.step(a, g.src, g.dst, g.ts, g.edge_feat, W, first, 40, neg, w.num_neighbors, w.num_heads, ix, deferred)
        rb = G.step(b, g.src, g.dst, g.ts, g.edge_feat, W, first, 40, neg, w.num_neighbors, w.num_heads,
                    G.Modules(), ix, deferred)
        for k in ("emb", "score_pos", "score_neg", "nbr_node", "nbr_eid", "nbr_ts", "nbr_cnt", "is_winner"):
            assert np.array_equal(ra[k], rb[k]), k
        assert np.array_equal(a.mem, b.mem) and np.array_equal(a.last_update, b.last_update)


def test_mean_equals_last_when_no_node_repeats():
    """A batch of two events whose four endpoints are distinct: one message per node."""
    src, dst, ts, feat = _graph()
    src, dst = src.copy(), dst.copy()
    src[4], dst[4], src[5], dst[5] = 0, 1, 2, 3
    rng = np.random.default_rng(5)
    W = {k: rng.normal(size=s).astype(np.float32) * 0.3 for k, s in S.weight_shapes(M, T, F, 2).items()}
    a, b = _state(), _state()
    ra = G.step(a, src, dst, ts, feat, W, 4, 2, None, 2, 2, G.Modules(aggregator="last"))
    rb = G.step(b, src, dst, ts, feat, W, 4, 2, None, 2, 2, G.Modules(aggregator="mean"))
    assert np.array_equal(a.mem, b.mem) and np.array_equal(a.last_update, b.last_update)
    assert np.array_equal(ra["emb"], rb["emb"])


# ------------------------------------------------------------------ mean aggregator by hand

@pytest.mark.parametrize("sel", range(D_MSG))
def test_mean_of_three_messages_by_hand(sel):
    """Batch = events 4 (0->1, t=10), 5 (2->0, t=12), 6 (0->3, t=15): node 0 has three messages
    (source, destination, source).  An RNN whose W_i row 0 selects message entry `sel` writes
    tanh(mean message[sel]) into memory entry 0; the three messages are written out here."""
    src, dst, ts, feat = _graph()
    W = _weights("rnn", "identity")
    W["W_i"][0, sel] = 1.0
    st = _state()
    mem0, lu0 = st.mem.copy(), st.last_update.copy()
    G.step(st, src, dst, ts, feat, W, 4, 3, None, 2, 2, G.Modules("mean", "rnn", "identity"))
    m0 = [np.concatenate([mem0[0], mem0[1], _phi(W, 10.0 - lu0[0]), feat[4]]),
          np.concatenate([mem0[0], mem0[2], _phi(W, 12.0 - lu0[0]), feat[5]]),
          np.concatenate([mem0[0], mem0[3], _phi(W, 15.0 - lu0[0]), feat[6]])]
    mean0 = np.float32((float(m0[0][sel]) + float(m0[1][sel]) + float(m0[2][sel])) / 3.0)
    assert st.mem[0, 0] == np.float32(math.tanh(float(mean0)))
    assert st.mem[0, 1] == 0.0
    # node 3: one message (destination of event 6); node 1, 2 likewise one each
    m3 = np.concatenate([mem0[3], mem0[0], _phi(W, 15.0 - lu0[3]), feat[6]])
    assert st.mem[3, 0] == np.float32(math.tanh(float(m3[sel])))
    assert st.last_update.tolist() == [15.0, 10.0, 12.0, 15.0]


def test_mean_differs_from_last_when_a_node_repeats():
    src, dst, ts, feat = _graph()
    W = _weights("rnn", "identity")
    W["W_i"][0, M] = 1.0     # partner's memory entry 0
    a, b = _state(), _state()
    G.step(a, src, dst, ts, feat, W, 4, 3, None, 2, 2, G.Modules("mean", "rnn", "identity"))
    G.step(b, src, dst, ts, feat, W, 4, 3, None, 2, 2, G.Modules("last", "rnn", "identity"))
    assert a.mem[0, 0] != b.mem[0, 0]
    assert np.array_equal(a.mem[1:3], b.mem[1:3])


def test_mean_does_not_depend_on_the_order_of_a_nodes_messages():
    msgs = [(7, 1.0, 3, np.array([1.0, 2.0], np.float32)), (7, 2.0, 4, np.array([0.5, -1.0], np.float32)),
            (7, 2.0, 5, np.array([3.0, 0.25], np.float32)), (2, 2.0, 5, np.array([9.0, 9.0], np.float32))]
    a = G.aggregate(msgs, "mean")
    b = G.aggregate(msgs[::-1], "mean")
    assert np.array_equal(a[7][0], np.array([1.5, 1.25 / 3.0], np.float32)) and a[7][1] == 2.0
    assert np.array_equal(a[7][0], b[7][0]) and np.array_equal(a[2][0], b[2][0])
    last = G.aggregate(msgs, "last")
    assert np.array_equal(last[7][0], msgs[2][3])      # (2.0, event 5) beats (2.0, event 4)


# ------------------------------------------------------------------ RNN cell

def test_rnn_closed_forms():
    m, h = np.array([0.3, -0.7, 1.1], np.float32), np.array([0.2, -0.4], np.float32)
    Z = lambda *s: np.zeros(s, np.float32)
    assert np.allclose(G.rnn_cell(m, h, Z(2, 3), np.array([0.5, -0.25], np.float32), Z(2, 2), Z(2)),
                       [math.tanh(0.5), math.tanh(-0.25)], rtol=0, atol=1e-15)
    Wi = np.array([[1, 0, 0], [0, 0, 2]], np.float32)
    Wh = np.array([[0, 1], [1, 0]], np.float32)
    got = G.rnn_cell(m, h, Wi, Z(2), Wh, np.array([0.0, 0.125], np.float32))
    want = [math.tanh(float(m[0]) + float(h[1])), math.tanh(2 * float(m[2]) + float(h[0]) + 0.125)]
    assert np.allclose(got, want, rtol=0, atol=1e-15)


def test_rnn_equals_library_cell_float64():
    rng = np.random.default_rng(3)
    D, Mm = 9, 5
    Wi, bi = rng.normal(size=(Mm, D)).astype(np.float32), rng.normal(size=Mm).astype(np.float32)
    Wh, bh = rng.normal(size=(Mm, Mm)).astype(np.float32), rng.normal(size=Mm).astype(np.float32)
    m, h = rng.normal(size=D).astype(np.float32), rng.normal(size=Mm).astype(np.float32)
    cell = torch.nn.RNNCell(D, Mm, nonlinearity="tanh").double()
    with torch.no_grad():
        cell.weight_ih.copy_(torch.from_numpy(Wi).double())
        cell.weight_hh.copy_(torch.from_numpy(Wh).double())
        cell.bias_ih.copy_(torch.from_numpy(bi).double())
        cell.bias_hh.copy_(torch.from_numpy(bh).double())
        want = cell(torch.from_numpy(m).double()[None], torch.from_numpy(h).double()[None])[0].numpy()
    assert np.allclose(G.rnn_cell(m, h, Wi, bi, Wh, bh), want, rtol=0, atol=1e-14)


# ------------------------------------------------------------------ identity / time projection / node features

def _pass_through_decoder(W, a_idx, b_idx):
    """score = relu(emb_a[a_idx]) - relu(-emb_a[a_idx]) + same for emb_b[b_idx]: the two entries, summed."""
    E = W["W_d1"].shape[0]
    W["W_d1"][:] = 0
    W["W_d1"][0, a_idx], W["W_d1"][1, a_idx] = 1.0, -1.0
    W["w_d2"][:] = 0
    W["w_d2"][0], W["w_d2"][1] = 1.0, -1.0
    assert E >= 2


def test_identity_embedding_is_the_updated_memory_row():
    src, dst, ts, feat = _graph()
    W = _weights("rnn", "identity")
    W["b_i"][:] = [0.4, -0.2]
    _pass_through_decoder(W, 1, 0)
    st = _state()
    mem0 = st.mem.copy()
    neg = np.array([3, 3], dtype=np.int32)
    out = G.step(st, src, dst, ts, feat, W, 4, 2, neg, 2, 2, G.Modules("last", "rnn", "identity"))
    new = np.array([math.tanh(0.4), math.tanh(-0.2)], dtype=np.float32)     # rows of nodes 0, 1, 2 after the step
    assert np.array_equal(st.mem[[0, 1, 2]], np.stack([new] * 3)) and np.array_equal(st.mem[3], mem0[3])
    want = np.stack([new, new, new, new, mem0[3], mem0[3]])                 # [src | dst | neg] rows
    assert np.array_equal(out["emb"], want)
    assert out["score_pos"].tolist() == [new[1], new[1]]                    # entry 1 of the source embedding
    assert out["nbr_cnt"] is None


def test_time_projection_by_hand():
    """Untouched node 3 queried as a negative at t = 10 and 12: (1 + (t - 4) * w_p) * memory; nodes
    updated by the step have dt = 0 only if their last event is the query's own."""
    src, dst, ts, feat = _graph()
    W = _weights("rnn", "time_projection")
    st = _state()
    mem0 = st.mem.copy()
    neg = np.array([3, 3], dtype=np.int32)
    out = G.step(st, src, dst, ts, feat, W, 4, 2, neg, 2, 2, G.Modules("last", "rnn", "time_projection"))
    wp = W["time_proj_w"].astype(np.float64)
    for b, t in ((0, 10.0), (1, 12.0)):
        want = ((1.0 + (t - 4.0) * wp) * mem0[3].astype(np.float64)).astype(np.float32)
        assert np.array_equal(out["emb"][4 + b], want)
    # all-zero RNN: updated rows are tanh(0) = 0 whatever the projection
    assert np.array_equal(out["emb"][:4], np.zeros((4, M), np.float32))
    # node 0 was last updated at t = 12 (event 5); its query of event 4 is at t = 10: dt = -2
    W["b_i"][:] = [0.4, -0.2]
    st = _state()
    out = G.step(st, src, dst, ts, feat, W, 4, 2, neg, 2, 2, G.Modules("last", "rnn", "time_projection"))
    new = np.array([math.tanh(0.4), math.tanh(-0.2)], dtype=np.float32).astype(np.float64)
    assert np.array_equal(out["emb"][0], ((1.0 + (10.0 - 12.0) * wp) * new).astype(np.float32))   # source of event 4
    assert np.array_equal(out["emb"][1], new.astype(np.float32))                                 # source of event 5: node 2, dt = 0
    zero_w = dict(W, time_proj_w=np.zeros(M, np.float32))
    st2 = _state()
    o2 = G.step(st2, src, dst, ts, feat, zero_w, 4, 2, neg, 2, 2, G.Modules("last", "rnn", "time_projection"))
    st3 = _state()
    o3 = G.step(st3, src, dst, ts, feat, zero_w, 4, 2, neg, 2, 2, G.Modules("last", "rnn", "identity"))
    assert np.array_equal(o2["emb"], o3["emb"])


def test_node_features_enter_the_embedding_not_the_message():
    src, dst, ts, feat = _graph()
    W = _weights("rnn", "identity")
    W["W_i"][0, 0] = 1.0     # own memory entry 0 -> would show a feature leaking into the message
    nf = np.array([[1, 2], [3, 4], [5, 6], [7, 8]], dtype=np.float32)
    a, b = _state(), _state()
    oa = G.step(a, src, dst, ts, feat, W, 4, 2, None, 2, 2, G.Modules("last", "rnn", "identity", nf))
    ob = G.step(b, src, dst, ts, feat, W, 4, 2, None, 2, 2, G.Modules("last", "rnn", "identity"))
    assert np.array_equal(a.mem, b.mem)
    q = oa["q_node"]
    assert np.array_equal(oa["emb"], (ob["emb"].astype(np.float64) + nf[q]).astype(np.float32))


def test_zero_node_features_change_nothing_and_attention_reads_them_for_neighbours():
    w = S.WORKLOADS["c1_tiny"]
    g, W = S.make_graph(w), S.make_weights(w)
    ix = O.NeighbourIndex(g.num_nodes, g.src, g.dst, g.ts)
    warm = S.make_warm_state(w, g, 5000)
    neg = S.make_negatives(w, g, 5000, 30)
    outs = []
    nf1 = S.make_node_feat(w, g.num_nodes)
    for nf in (None, np.zeros((g.num_nodes, w.mem_dim), np.float32), nf1):
        st = O.OracleState(warm[0].copy(), warm[1].copy())
        outs.append((G.step(st, g.src, g.dst, g.ts, g.edge_feat, W, 5000, 30, neg, w.num_neighbors, w.num_heads,
                            G.Modules(node_feat=nf), ix), st))
    assert np.array_equal(outs[0][0]["emb"], outs[1][0]["emb"])
    assert np.array_equal(outs[0][1].mem, outs[2][1].mem)          # memory never sees node features
    # adding v to every memory row by hand and running without features gives the same embeddings
    # once the update is switched off (z = 1 keeps the state): r = s + v either way
    Wk = dict(W)
    Wk["b_i"] = W["b_i"].copy()
    Wk["b_i"][w.mem_dim:2 * w.mem_dim] = 400.0
    st_a = O.OracleState(warm[0].copy(), warm[1].copy())
    oa = G.step(st_a, g.src, g.dst, g.ts, g.edge_feat, Wk, 5000, 30, neg, w.num_neighbors, w.num_heads,
                G.Modules(node_feat=nf1), ix)
    st_b = O.OracleState((warm[0].astype(np.float64) + nf1).astype(np.float32), warm[1].copy())
    ob = O.step(st_b, g.src, g.dst, g.ts, g.edge_feat, Wk, 5000, 30, neg, w.num_neighbors, w.num_heads, ix)
    assert np.array_equal(oa["emb"], ob["emb"])


def test_deferred_order_applies_the_previous_batch():
    """Memory after deferred steps over b1, b2 equals memory after the update-first step over b1."""
    src, dst, ts, feat = _graph()
    W = _weights("rnn", "identity")
    W["W_i"][0, M] = 1.0
    W["b_i"][:] = [0.1, 0.2]
    mods = G.Modules("mean", "rnn", "identity")
    a, b = _state(), _state()
    G.step(a, src, dst, ts, feat, W, 2, 2, None, 2, 2, mods, deferred=True)
    assert np.array_equal(a.mem, b.mem)                      # the first deferred step applies nothing
    G.step(a, src, dst, ts, feat, W, 4, 3, None, 2, 2, mods, deferred=True)
    G.step(b, src, dst, ts, feat, W, 2, 2, None, 2, 2, mods)
    assert np.array_equal(a.mem, b.mem) and np.array_equal(a.last_update, b.last_update)
