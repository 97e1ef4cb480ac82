"""CPU oracle of the batch step for OTHER INSTANCES of the general architecture.  TEST
INFRASTRUCTURE ONLY: imported by tests, the smoke check and the benchmark's CPU-baseline leg.

The paper's Sec. II-C ("Training approach for TIGs") states the encoder as four modules with
interchangeable parts: messages of a node within a batch "can be aggregated by ... mean message or
other" functions, the state update "can be chosen from ... GRU, RNN", and the embedding function f
is "identity, time projection or attention"; Sec. II-A gives nodes optional static features.  The
batch step of oracle/tig_oracle.py fixes one instance (last message, GRU, attention, no node
features); this file states the step for the others, in float64 NumPy on float32 inputs, rounded to
float32 only where the method stores a value:

  AGG  "last"   the node's message with the greatest (time, event id)      (tig_oracle)
       "mean"   the element-wise mean of ALL the node's messages of the batch, either role, each
                built from the memory at the start of the step with its own event's time, partner
                and feature row; the node's last_update becomes the time of its last event
  UPD  "gru"    tig_oracle.gru_cell
       "rnn"    s = tanh(W_i m + b_i + W_h s' + b_h)                        (W_i [M, D_msg], W_h [M, M])
  f    "attention"        tig_oracle.attention + merge over the K most recent neighbours
       "identity"         emb_i(t) = r_i(t)                                 (E = M, no neighbours read)
       "time_projection"  emb_i(t) = (1 + (t - last_update_i) * w_p) * r_i(t), w_p [M], with the
                          last_update the step's memory overwrite left     (E = M)
  node features v [N, M]: wherever the embedding module reads a node's state -- its own or a
       neighbour's -- it reads r_i(t) = s_i(t) + v_i; messages carry the raw memory rows.
  layers  the embedding sums over the k-hop temporal neighbourhood neighbor_i^k([0, t]) (Sec. II-C,
       embedding module).  With the attention function, k = 2 is two stacked layers:
         h0_i(t) = r_i(t)
         hl_i(t) = merge_l(attention_l([h(l-1)_i(t) | Phi(0)], {[h(l-1)_j(t) | e_ij | Phi(t - t_ij)]}), h(l-1)_i(t))
       over the K most recent neighbours j of i before t.  Every row of layer l-1 is taken AT THE
       QUERY TIME t: a neighbour's layer-1 row attends over that neighbour's own K most recent
       events before t (which include its event with i).  Layer 1 has the weights of the one-layer
       model; layer 2 has a set of its own, with the layer-1 width E where layer 1 has the state
       width M: W_Q, W_O [E+T, E+T], W_K, W_V [E+T, E+F+T], W_m1 [E, 2E+T], W_m2 [E, E].

These details are this build's readings (the paper names the options and gives no formulas):
parity unpinned for the CHOICES.  The implementation of each is pinned in
tests/test_modules_oracle.py: reduction to tig_oracle.step bit for bit when the instance is the
headline one; mean == last when no node repeats in a batch; a hand-worked three-message mean seen
through selector weights; order independence of the mean; the RNN cell against closed forms and the
float64 library cell; identity / time-projection values written out by hand; zero node features ==
no node features; two layers: a pass-through second layer returns the first layer's rows, a
second layer that averages its neighbour rows returns the mean of the one-layer embeddings that
the pinned one-layer step gives for those neighbours as negatives at the query's time, a chain
graph whose far end is visible only through the second hop, no future event within either hop.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from . import tig_oracle as O

f32 = np.float32
f64 = np.float64


@dataclass
class Modules:
    aggregator: str = "last"         # "last" | "mean"
    updater: str = "gru"             # "gru" | "rnn"
    embedding: str = "attention"     # "attention" | "identity" | "time_projection"
    node_feat: np.ndarray = None     # float32 [N, M] or None
    layers: int = 1                  # attention embedding: 1 or 2 stacked layers
    layer2: dict = None              # weights of the second layer (W_Q b_Q W_K b_K W_V b_V W_O b_O W_m1 b_m1 W_m2 b_m2)


def rnn_cell(m, h, W_i, b_i, W_h, b_h):
    """State update UPD(s', m) of Sec. II-C as a plain recurrent cell: tanh(W_i m + b_i + W_h s' + b_h)."""
    return np.tanh(W_i.astype(f64) @ m.astype(f64) + b_i.astype(f64) + W_h.astype(f64) @ h.astype(f64) + b_h.astype(f64))


def messages_of_batch(mem0, lu0, s_b, d_b, t_b, eids, edge_feat, W):
    """Every message of a batch: for event b and role (0 source, 1 destination) the row
    [s'_self | s'_other | Phi(t_b - last_update[self]) | e_b], float32, from the memory (mem0, lu0) at
    the start of the step.  Returns a list of (node, time, event id, message) in (event, role) order."""
    out = []
    for b in range(len(eids)):
        for u, o in ((int(s_b[b]), int(d_b[b])), (int(d_b[b]), int(s_b[b]))):
            phi = O.time_encode(float(t_b[b]) - lu0[u], W["time_w"], W["time_b"])
            msg = np.concatenate([mem0[u], mem0[o], phi, edge_feat[int(eids[b])]]).astype(f32)
            out.append((u, float(t_b[b]), int(eids[b]), msg))
    return out


def aggregate(msgs, how):
    """{node: (aggregated message float32, time of the node's last event)}.  "mean": element-wise mean
    of the node's messages, summed in float64, stored float32; "last": greatest (time, event id)."""
    per_node = {}
    for u, t, eid, m in msgs:
        per_node.setdefault(u, []).append((t, eid, m))
    agg = {}
    for u, lst in per_node.items():
        t_last, _, m_last = max(lst, key=lambda x: (x[0], x[1]))
        if how == "mean":
            mean = np.sum([m.astype(f64) for _, _, m in lst], axis=0) / float(len(lst))
            agg[u] = (mean.astype(f32), t_last)
        else:
            agg[u] = (m_last, t_last)
    return agg


def apply_batch(state, src, dst, ts, edge_feat, W, first_eid, count, mods):
    """Message, aggregation, state update and memory overwrite for the events first_eid ..
    first_eid + count - 1, every message built from the memory as it stands at the start of the call."""
    if count <= 0:
        return
    eids = np.arange(first_eid, first_eid + count)
    mem0 = state.mem.copy()
    lu0 = state.last_update.copy()
    msgs = messages_of_batch(mem0, lu0, src[eids], dst[eids], ts[eids], eids, edge_feat, W)
    for u, (m, t_last) in aggregate(msgs, mods.aggregator).items():
        if mods.updater == "rnn":
            h_new = rnn_cell(m, mem0[u], W["W_i"], W["b_i"], W["W_h"], W["b_h"])
        else:
            h_new = O.gru_cell(m, mem0[u], W["W_i"], W["b_i"], W["W_h"], W["b_h"])
        state.mem[u] = h_new.astype(f32)
        state.last_update[u] = t_last


def node_repr(state, mods, u):
    """r_i(t): the state the embedding module reads for node i (memory row, plus the static feature row)."""
    r = state.mem[u].astype(f64)
    if mods.node_feat is not None:
        r = r + mods.node_feat[u].astype(f64)
    return r.astype(f32)


def embed_layer(state, mods, W, edge_feat, H, lookup, l, u, t, table=None):
    """h^l_u(t) of the attention embedding (float32 [M] for l = 0, [E] above): layer l over the K most
    recent neighbours of u before t, every input row being the layer l-1 row of its node at the SAME
    time t.  lookup(nodes, times) -> (nbr_node, nbr_eid, nbr_ts, nbr_cnt); table: the row of that
    answer for (u, t) if the caller has it already."""
    if l == 0:
        return node_repr(state, mods, u)
    Wl = W if l == 1 else mods.layer2
    if table is None:
        nn, ne, nt, nc = lookup(np.array([u], dtype=np.int32), np.array([t], dtype=f64))
        table = (nn[0], ne[0], nt[0], int(nc[0]))
    nb_node, nb_eid, nb_ts, c = table
    h_self = embed_layer(state, mods, W, edge_feat, H, lookup, l - 1, u, t)
    q_in = np.concatenate([h_self, O.time_encode(0.0, W["time_w"], W["time_b"])])
    if c > 0:
        h_nb = np.stack([embed_layer(state, mods, W, edge_feat, H, lookup, l - 1, int(v), t) for v in nb_node[:c]])
        phi_k = O.time_encode(t - nb_ts[:c], W["time_w"], W["time_b"])
        kv = np.concatenate([h_nb, edge_feat[nb_eid[:c]], phi_k], axis=1).astype(f32)
    else:
        kv = np.zeros((0, h_self.shape[0] + edge_feat.shape[1] + W["time_w"].shape[0]), dtype=f32)
    return O.merge(O.attention(q_in, kv, Wl, H), h_self, Wl).astype(f32)


def step(state, src, dst, ts, edge_feat, W, first_eid, count, neg_dst, K, H, mods, index=None, deferred=False):
    """One chronological batch step of the chosen instance; updates `state` in place.  Same outputs
    and conventions as tig_oracle.step (neighbour tables only for the attention embedding).
    state.pending holds (first_eid, count) of the batch kept by a deferred step, or []."""
    eids = np.arange(first_eid, first_eid + count)
    s_b, d_b, t_b = src[eids], dst[eids], ts[eids]
    win = O.find_winners(s_b, d_b, t_b, eids)
    is_winner = np.zeros(2 * count, dtype=np.uint8)
    for u, (b, role) in win.items():
        is_winner[2 * b + role] = 1

    if deferred:
        if state.pending:
            apply_batch(state, src, dst, ts, edge_feat, W, state.pending[0], state.pending[1], mods)
        state.pending = [first_eid, count]
    else:
        apply_batch(state, src, dst, ts, edge_feat, W, first_eid, count, mods)
        state.pending = []

    if neg_dst is not None:
        q_node = np.concatenate([s_b, d_b, np.asarray(neg_dst, dtype=np.int32)])
        q_time = np.concatenate([t_b, t_b, t_b])
    else:
        q_node = np.concatenate([s_b, d_b])
        q_time = np.concatenate([t_b, t_b])
    Q = q_node.shape[0]
    M = state.mem.shape[1]
    res = {"q_node": q_node, "q_time": q_time, "is_winner": is_winner,
           "nbr_node": None, "nbr_eid": None, "nbr_ts": None, "nbr_cnt": None}

    if mods.embedding == "attention":
        if index is None:
            lookup = lambda nodes, times: O.neighbours_bruteforce_batch(src, dst, ts, nodes, times, K)
        else:
            lookup = lambda nodes, times: index.query(nodes, times, K)
        nb_node, nb_eid, nb_ts, nb_cnt = lookup(q_node, q_time)
        res.update(nbr_node=nb_node, nbr_eid=nb_eid, nbr_ts=nb_ts, nbr_cnt=nb_cnt)
        E = W["W_m2"].shape[0]
        emb = np.empty((Q, E), dtype=f32)
        for q in range(Q):
            table = (nb_node[q], nb_eid[q], nb_ts[q], int(nb_cnt[q]))
            emb[q] = embed_layer(state, mods, W, edge_feat, H, lookup, mods.layers, int(q_node[q]), float(q_time[q]), table)
    else:
        emb = np.empty((Q, M), dtype=f32)
        for q in range(Q):
            u = int(q_node[q])
            r_u = node_repr(state, mods, u).astype(f64)
            if mods.embedding == "time_projection":
                dt = float(q_time[q]) - float(state.last_update[u])
                r_u = (1.0 + dt * W["time_proj_w"].astype(f64)) * r_u
            emb[q] = r_u.astype(f32)

    score_pos = np.empty(count, dtype=f32)
    score_neg = np.empty(count, dtype=f32) if neg_dst is not None else None
    for b in range(count):
        score_pos[b] = O.decoder(emb[b], emb[count + b], W)
        if neg_dst is not None:
            score_neg[b] = O.decoder(emb[b], emb[2 * count + b], W)
    res.update(emb=emb, score_pos=score_pos, score_neg=score_neg)
    return res
