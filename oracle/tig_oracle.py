"""CPU oracle of the TIG batch step.  TEST INFRASTRUCTURE ONLY.

A plain, slow, float64 NumPy statement of what one chronological mini-batch
step of a memory-based temporal-interaction-graph model computes, following
the encoder/decoder data flow in the paper's Sec. II-C ("Training approach for
TIGs"): memory fetch -> message -> per-node aggregation -> state update ->
memory overwrite -> neighbour embedding -> pairwise decoder.

It is imported only by tests, by the smoke check and by the benchmark's
CPU-baseline leg.  It shares no code with the GPU library and never imports it.

Instance of the paper's general architecture that is computed here
(the paper leaves these choices open; they are fixed by this build):
  MSG   = concatenation [s'_self | s'_other | Phi(dt) | e_ij(t)]
  AGG   = last message of the node in the batch, "last" by (time, event id)
  UPD   = GRU cell (gates r, z, n; reset gate applied to the hidden product)
  f     = one layer of multi-head scaled-dot-product attention over the K most
          recent neighbours, followed by a two-layer merge MLP
  g     = two-layer MLP on the concatenated pair of embeddings (raw logit)
  Phi   = cos(w * x + b)   (the time encoding the paper cites)

Precision: float64 arithmetic on float32 inputs; a value is rounded to float32
only where the method stores it (message entries, memory rows, key/value
entries, embeddings, scores).

Pins (tests/test_oracle_*.py): brute-force neighbour definition vs an
independent sort, hand-built tie cases, closed forms of the GRU and attention,
library GRU cell and library scaled-dot-product attention in float64,
whole-step invariants (untouched rows, no future leakage, batch-order
independence).  The architecture choices themselves (update-before-embed order,
GRU variant, attention widths, empty-neighbourhood rule, initialisation) are
fixed by this build, not by the paper: parity unpinned for those choices.

Deferred order (step(..., deferred=True)): the step first applies the winners
that the PREVIOUS step kept (messages built from the memory as it stands now),
then embeds, then keeps its own batch's winners for the next step -- the order a
training loop uses so that a prediction never sees its own event through the
memory.  Pins: the memory after deferred steps over batches b1, b2 equals the
memory after the update-first step over b1; with a GRU that keeps the state
(z = 1) both orders give the same embeddings; the first step after a reset
applies nothing.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_NBR_SRC = os.path.join(_HERE, "nbr_index.c")
_NBR_LIB = os.path.join(_HERE, "liboracle_nbr.so")

f32 = np.float32
f64 = np.float64


# --------------------------------------------------------------------------- building blocks


def time_encode(x, w, b):
    """Phi(x)_k = cos(w_k * x + b_k)  (time encoding used in the message and in the
    attention keys, Sec. II-C).  w, b are float32 parameters, x float64 time differences.
    Evaluated in float64, stored as float32.  x may be a scalar or an array [...]; result
    has shape [..., T]."""
    x = np.asarray(x, dtype=f64)
    arg = x[..., None] * w.astype(f64) + b.astype(f64)
    return np.cos(arg).astype(f32)


def sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def find_winners(nodes_src, nodes_dst, times, eids):
    """Last-message aggregation (Sec. II-C: all messages of a node within one batch are
    aggregated; this build keeps the last one).  For every node that occurs in the batch,
    the occurrence with the lexicographically greatest (time, event id) wins.

    Returns {node: (b, role)} with b the position in the batch and role 0 = source,
    1 = destination."""
    best = {}
    for b in range(len(eids)):
        for role, u in ((0, int(nodes_src[b])), (1, int(nodes_dst[b]))):
            key = (float(times[b]), int(eids[b]))
            if u not in best or key > best[u][0]:
                best[u] = (key, b, role)
    return {u: (v[1], v[2]) for u, v in best.items()}


def gru_cell(m, h, W_i, b_i, W_h, b_h):
    """State update UPD(s', m) of Sec. II-C as a GRU cell.  Gates stacked (r, z, n) in
    W_i [3M, D_msg], W_h [3M, M]:
        r = sig(W_ir m + b_ir + W_hr h + b_hr)
        z = sig(W_iz m + b_iz + W_hz h + b_hz)
        n = tanh(W_in m + b_in + r * (W_hn h + b_hn))
        h' = (1 - z) * n + z * h
    All float64; returns float64 [M]."""
    M = h.shape[0]
    m = m.astype(f64)
    h = h.astype(f64)
    gi = W_i.astype(f64) @ m + b_i.astype(f64)
    gh = W_h.astype(f64) @ h + b_h.astype(f64)
    r = sigmoid(gi[0:M] + gh[0:M])
    z = sigmoid(gi[M:2 * M] + gh[M:2 * M])
    n = np.tanh(gi[2 * M:3 * M] + r * gh[2 * M:3 * M])
    return (1.0 - z) * n + z * h


def neighbours_bruteforce(src, dst, ts, u, t, K):
    """Most-recent-K temporal neighbours of node u before time t, by definition:
    scan every event of the graph, keep those incident to u whose time is strictly
    earlier than t (the history E_t of the Notations section), and take the K greatest by
    (time, event id).  Slot 0 is the most recent; unused slots are (-1, -1, 0.0)."""
    incident = (src == u) | (dst == u)
    cand = np.flatnonzero(incident & (ts < t))
    order = np.lexsort((cand, ts[cand]))          # ascending by (time, event id)
    top = cand[order][::-1][:K]                   # descending, K most recent
    nb_node = np.full(K, -1, dtype=np.int32)
    nb_eid = np.full(K, -1, dtype=np.int32)
    nb_ts = np.zeros(K, dtype=f64)
    for k, e in enumerate(top):
        nb_eid[k] = e
        nb_node[k] = dst[e] if src[e] == u else src[e]
        nb_ts[k] = ts[e]
    return nb_node, nb_eid, nb_ts, len(top)


def attention(q_in, kv, W, H):
    """One layer of H-head scaled-dot-product attention of a query vector q_in [d_a] over
    cnt key/value rows kv [cnt, d_kv] (the "attention" choice of the embedding function f,
    Sec. II-C).  Heads are contiguous slices of width d_h = d_a / H.  Softmax runs over the
    cnt rows only.  An empty neighbourhood gives the zero vector.  float64 in and out."""
    d_a = W["W_Q"].shape[0]
    if kv.shape[0] == 0:
        return np.zeros(d_a, dtype=f64)
    d_h = d_a // H
    Qv = W["W_Q"].astype(f64) @ q_in.astype(f64) + W["b_Q"].astype(f64)
    Kp = kv.astype(f64) @ W["W_K"].astype(f64).T + W["b_K"].astype(f64)    # [cnt, d_a]
    Vp = kv.astype(f64) @ W["W_V"].astype(f64).T + W["b_V"].astype(f64)    # [cnt, d_a]
    out = np.zeros(d_a, dtype=f64)
    for h in range(H):
        sl = slice(h * d_h, (h + 1) * d_h)
        s = Kp[:, sl] @ Qv[sl] / np.sqrt(float(d_h))
        s = s - s.max()
        a = np.exp(s)
        a = a / a.sum()
        out[sl] = a @ Vp[:, sl]
    return W["W_O"].astype(f64) @ out + W["b_O"].astype(f64)


def merge(attn, mem_u, W):
    """emb = W_m2 relu(W_m1 [attn | s_u] + b_m1) + b_m2  (learnable part of f)."""
    x = np.concatenate([attn.astype(f64), mem_u.astype(f64)])
    hid = np.maximum(W["W_m1"].astype(f64) @ x + W["b_m1"].astype(f64), 0.0)
    return W["W_m2"].astype(f64) @ hid + W["b_m2"].astype(f64)


def decoder(emb_a, emb_b, W):
    """g(emb_a, emb_b): logit = w_d2 . relu(W_d1 [emb_a | emb_b] + b_d1) + b_d2."""
    x = np.concatenate([emb_a.astype(f64), emb_b.astype(f64)])
    hid = np.maximum(W["W_d1"].astype(f64) @ x + W["b_d1"].astype(f64), 0.0)
    return float(W["w_d2"].astype(f64) @ hid + W["b_d2"].astype(f64)[0])


# --------------------------------------------------------------------------- indexed neighbours


def build_native(force: bool = True) -> str:
    """Compile the indexed neighbour routine (plain C, single thread)."""
    if force or not os.path.exists(_NBR_LIB):
        subprocess.run(["gcc", "-O2", "-fPIC", "-shared", "-fvisibility=hidden", "-std=c11", "-o",
                        _NBR_LIB, _NBR_SRC], check=True)
    return _NBR_LIB


class NeighbourIndex:
    """Per-node time-ordered event lists + binary search (oracle/nbr_index.c).  Used where
    the brute-force scan is unaffordable; checked bit-for-bit against it in the tests."""

    def __init__(self, num_nodes, src, dst, ts):
        if not os.path.exists(_NBR_LIB):
            build_native(force=True)
        lib = ctypes.CDLL(_NBR_LIB)
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
        lib.nbr_index_build.restype = vp
        lib.nbr_index_build.argtypes = [i64, i64, vp, vp, vp]
        lib.nbr_index_free.argtypes = [vp]
        lib.nbr_index_free.restype = None
        lib.nbr_index_query.restype = ctypes.c_int
        lib.nbr_index_query.argtypes = [vp, i64, vp, vp, i32, vp, vp, vp, vp]
        self._lib = lib
        self._keep = (np.ascontiguousarray(src, dtype=np.int32),
                      np.ascontiguousarray(dst, dtype=np.int32),
                      np.ascontiguousarray(ts, dtype=f64))
        self._h = lib.nbr_index_build(int(num_nodes), int(self._keep[0].shape[0]),
                                      self._keep[0].ctypes.data, self._keep[1].ctypes.data,
                                      self._keep[2].ctypes.data)
        if not self._h:
            raise ValueError("nbr_index_build failed (ids out of range or unsorted times)")

    def query(self, nodes, times, K):
        nodes = np.ascontiguousarray(nodes, dtype=np.int32)
        times = np.ascontiguousarray(times, dtype=f64)
        Q = nodes.shape[0]
        nb_node = np.empty((Q, K), dtype=np.int32)
        nb_eid = np.empty((Q, K), dtype=np.int32)
        nb_ts = np.empty((Q, K), dtype=f64)
        cnt = np.empty(Q, dtype=np.int32)
        rc = self._lib.nbr_index_query(self._h, Q, nodes.ctypes.data, times.ctypes.data, int(K),
                                       nb_node.ctypes.data, nb_eid.ctypes.data, nb_ts.ctypes.data,
                                       cnt.ctypes.data)
        if rc != 0:
            raise RuntimeError("nbr_index_query failed")
        return nb_node, nb_eid, nb_ts, cnt

    def __del__(self):
        try:
            if self._h:
                self._lib.nbr_index_free(self._h)
                self._h = None
        except Exception:
            pass


def neighbours_bruteforce_batch(src, dst, ts, nodes, times, K):
    Q = len(nodes)
    nb_node = np.empty((Q, K), dtype=np.int32)
    nb_eid = np.empty((Q, K), dtype=np.int32)
    nb_ts = np.empty((Q, K), dtype=f64)
    cnt = np.empty(Q, dtype=np.int32)
    for q in range(Q):
        nb_node[q], nb_eid[q], nb_ts[q], cnt[q] = neighbours_bruteforce(
            src, dst, ts, int(nodes[q]), float(times[q]), K)
    return nb_node, nb_eid, nb_ts, cnt


# --------------------------------------------------------------------------- the step


@dataclass
class OracleState:
    mem: np.ndarray          # float32 [N, M]   node memory (the memory module of Sec. II-C)
    last_update: np.ndarray  # float64 [N]      time of each node's last memory update
    # deferred order only: winners (node, partner, event id, time) kept for the next step
    pending: list = None

    def __post_init__(self):
        if self.pending is None:
            self.pending = []

    @staticmethod
    def zeros(num_nodes, mem_dim):
        """State after a reset (memory reset at the start of a data cycle, Alg. 2)."""
        return OracleState(np.zeros((num_nodes, mem_dim), dtype=f32),
                           np.zeros(num_nodes, dtype=f64))

    def copy(self):
        st = OracleState(self.mem.copy(), self.last_update.copy())
        st.pending = list(self.pending)
        return st

    def drop_pending(self):
        """What a reset or a restore of the memory does to the winners kept by a deferred step."""
        self.pending = []


def apply_messages(state, winners, edge_feat, W):
    """Message, state update and memory overwrite (MSG, UPD and M <- s_i(t) of Sec. II-C) for a
    list of (node, partner, event id, time); every message reads the memory as it stands at
    the start of the call."""
    mem0 = state.mem.copy()
    lu0 = state.last_update.copy()
    for u, other, eid, t in winners:
        phi = time_encode(t - lu0[u], W["time_w"], W["time_b"])
        msg = np.concatenate([mem0[u], mem0[other], phi, edge_feat[eid]]).astype(f32)
        h_new = gru_cell(msg, mem0[u], W["W_i"], W["b_i"], W["W_h"], W["b_h"])
        state.mem[u] = h_new.astype(f32)
        state.last_update[u] = t


def step(state, src, dst, ts, edge_feat, W, first_eid, count, neg_dst, K, H, index=None, deferred=False):
    """One chronological batch step; updates `state` in place and returns a dict with
    emb [Q, E], score_pos [count], score_neg [count] (or None), the neighbour tables, and
    is_winner [2*count] (entry 2*b + role).  Q = 3*count with negatives, else 2*count; query
    rows are ordered [sources | destinations | negatives].

    `index` is a NeighbourIndex over the same graph, or None for the brute-force scan."""
    M = state.mem.shape[1]
    eids = np.arange(first_eid, first_eid + count)
    s_b, d_b, t_b = src[eids], dst[eids], ts[eids]

    # 2. aggregation: last message per node
    win = find_winners(s_b, d_b, t_b, eids)
    is_winner = np.zeros(2 * count, dtype=np.uint8)
    winners = []
    for u, (b, role) in win.items():
        is_winner[2 * b + role] = 1
        other = int(d_b[b]) if role == 0 else int(s_b[b])
        winners.append((int(u), other, int(eids[b]), float(t_b[b])))

    # 1., 3.-5. previous states are fetched from the memory as it stands at the start of the
    # step; message, GRU update, overwrite memory -- for this batch's winners, or in the deferred
    # order for the winners the previous step kept (this batch's are kept for the next step)
    apply_messages(state, state.pending if deferred else winners, edge_feat, W)
    state.pending = winners if deferred else []

    # 6. neighbours of every query, from the whole graph, strictly before the query time
    if neg_dst is not None:
        q_node = np.concatenate([s_b, d_b, np.asarray(neg_dst, dtype=np.int32)])
        q_time = np.concatenate([t_b, t_b, t_b])
    else:
        q_node = np.concatenate([s_b, d_b])
        q_time = np.concatenate([t_b, t_b])
    if index is None:
        nb_node, nb_eid, nb_ts, nb_cnt = neighbours_bruteforce_batch(src, dst, ts, q_node, q_time, K)
    else:
        nb_node, nb_eid, nb_ts, nb_cnt = index.query(q_node, q_time, K)

    # 7.-8. attention over the neighbours with the UPDATED memory, then merge
    Q = q_node.shape[0]
    E = W["W_m2"].shape[0]
    emb = np.empty((Q, E), dtype=f32)
    phi0 = time_encode(0.0, W["time_w"], W["time_b"])
    for q in range(Q):
        u = int(q_node[q])
        c = int(nb_cnt[q])
        q_in = np.concatenate([state.mem[u], phi0])
        if c > 0:
            vs = nb_node[q, :c]
            phi_k = time_encode(q_time[q] - nb_ts[q, :c], W["time_w"], W["time_b"])
            kv = np.concatenate([state.mem[vs], edge_feat[nb_eid[q, :c]], phi_k], axis=1).astype(f32)
        else:
            kv = np.zeros((0, M + edge_feat.shape[1] + W["time_w"].shape[0]), dtype=f32)
        a = attention(q_in, kv, W, H)
        emb[q] = merge(a, state.mem[u], W).astype(f32)

    # 9. decoder on (source, destination) and (source, negative)
    score_pos = np.empty(count, dtype=f32)
    score_neg = np.empty(count, dtype=f32) if neg_dst is not None else None
    for b in range(count):
        score_pos[b] = decoder(emb[b], emb[count + b], W)
        if neg_dst is not None:
            score_neg[b] = decoder(emb[b], emb[2 * count + b], W)

    return {"emb": emb, "score_pos": score_pos, "score_neg": score_neg,
            "nbr_node": nb_node, "nbr_eid": nb_eid, "nbr_ts": nb_ts, "nbr_cnt": nb_cnt,
            "is_winner": is_winner, "q_node": q_node, "q_time": q_time}
