"""Pins of the training-step oracle (oracle/train_oracle.py): loss and hand-written backward pass
(Sec. II-C self-supervised signal; Alg. 2 "Backward and Optimize")."""
import math

import numpy as np
import pytest
import torch

import tig_synth as S
from oracle import tig_oracle as O
from oracle import train_oracle as T


@pytest.fixture(scope="module")
def c1():
    w = S.WORKLOADS["c1_tiny"]
    return w, S.make_graph(w), S.make_weights(w)


def warm(w, g, first):
    return O.OracleState(*S.make_warm_state(w, g, first))


def test_loss_closed_forms():
    z = np.zeros(5, dtype=np.float32)
    assert T.bce_loss(z, z) == pytest.approx(2 * math.log(2.0), rel=1e-15)
    assert T.bce_loss(np.full(3, 40.0, np.float32), np.full(3, -40.0, np.float32)) == pytest.approx(0.0, abs=1e-15)
    # a confident mistake costs its logit: softplus(x) -> x
    assert T.bce_loss(np.full(2, -30.0, np.float32), z[:2]) == pytest.approx(30.0 + math.log(2.0), rel=1e-12)
    p, n = np.array([0.3, -1.2], np.float32), np.array([0.7, 2.0], np.float32)
    want = -np.mean(np.log(1 / (1 + np.exp(-p.astype(float))))) - np.mean(np.log(1 - 1 / (1 + np.exp(-n.astype(float)))))
    assert T.bce_loss(p, n) == pytest.approx(want, rel=1e-14)


@pytest.mark.parametrize("deferred", [False, True])
def test_forward_is_the_batch_step_and_lr_zero_changes_nothing(c1, deferred):
    w, g, W = c1
    a, b = warm(w, g, 4000), warm(w, g, 4000)
    W2 = {k: v.copy() for k, v in W.items()}
    ix = O.NeighbourIndex(g.num_nodes, g.src, g.dst, g.ts)
    for first in (4000, 4060):
        neg = S.make_negatives(w, g, first, 60)
        ref = O.step(a, g.src, g.dst, g.ts, g.edge_feat, W, first, 60, neg, w.num_neighbors, w.num_heads, index=ix,
                     deferred=deferred)
        out, loss, grads = T.train_step(b, g.src, g.dst, g.ts, g.edge_feat, W2, first, 60, neg, w.num_neighbors,
                                        w.num_heads, 0.0, index=ix, deferred=deferred)
        for k in ("emb", "score_pos", "score_neg", "nbr_node", "is_winner"):
            assert np.array_equal(out[k], ref[k])
        assert np.array_equal(a.mem, b.mem) and np.array_equal(a.last_update, b.last_update)
        assert loss == T.bce_loss(ref["score_pos"], ref["score_neg"])
        assert all(np.array_equal(W[k], W2[k]) for k in W)
    assert any(np.abs(v).max() > 0 for v in grads.values())


def torch_loss(Wt, w, g, applied, before, post_mem, out, count):
    """The step's loss as a function of the weights, written with torch ops in float64: GRU of the
    applied winners from the rows they read (library GRU cell semantics via torch.nn.functional),
    attention and MLPs with plain tensor algebra."""
    M, T_, H = w.mem_dim, w.time_dim, w.num_heads
    t64 = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))
    new_rows = {}
    for u, other, eid, t in applied:
        mem_u, mem_o, lu_u = before[u]
        phi = torch.cos(Wt["time_w"] * (t - lu_u) + Wt["time_b"])
        m = torch.cat([t64(mem_u), t64(mem_o), phi, t64(g.edge_feat[eid])])
        cell = torch.nn.GRUCell(m.numel(), M, dtype=torch.float64)
        new_rows[u] = torch.func.functional_call(
            cell, {"weight_ih": Wt["W_i"], "weight_hh": Wt["W_h"], "bias_ih": Wt["b_i"], "bias_hh": Wt["b_h"]},
            (m[None], t64(mem_u)[None]))[0]
    row = lambda v: new_rows[v] if v in new_rows else t64(post_mem[v])
    d_a = M + T_
    d_h = d_a // H
    embs = []
    for q in range(out["emb"].shape[0]):
        u, c = int(out["q_node"][q]), int(out["nbr_cnt"][q])
        s_u = row(u)
        if c > 0:
            q_in = torch.cat([s_u, torch.cos(Wt["time_b"])])
            kv = torch.stack([torch.cat([row(int(out["nbr_node"][q, k])), t64(g.edge_feat[out["nbr_eid"][q, k]]),
                                         torch.cos(Wt["time_w"] * (out["q_time"][q] - out["nbr_ts"][q, k]) + Wt["time_b"])])
                              for k in range(c)])
            Q = (Wt["W_Q"] @ q_in + Wt["b_Q"]).view(H, d_h)
            Kp = (kv @ Wt["W_K"].T + Wt["b_K"]).view(c, H, d_h)
            Vp = (kv @ Wt["W_V"].T + Wt["b_V"]).view(c, H, d_h)
            a = torch.softmax(torch.einsum("khd,hd->hk", Kp, Q) / math.sqrt(d_h), dim=1)
            attn = Wt["W_O"] @ torch.einsum("hk,khd->hd", a, Vp).reshape(d_a) + Wt["b_O"]
        else:
            attn = torch.zeros(d_a, dtype=torch.float64)
        hid = torch.relu(Wt["W_m1"] @ torch.cat([attn, s_u]) + Wt["b_m1"])
        embs.append(Wt["W_m2"] @ hid + Wt["b_m2"])
    emb = torch.stack(embs)
    dec = lambda a, b: torch.relu(torch.cat([a, b], dim=1) @ Wt["W_d1"].T + Wt["b_d1"]) @ Wt["w_d2"] + Wt["b_d2"]
    pos = dec(emb[:count], emb[count:2 * count])
    neg = dec(emb[:count], emb[2 * count:])
    return torch.nn.functional.softplus(-pos).mean() + torch.nn.functional.softplus(neg).mean()


@pytest.mark.parametrize("deferred,first", [(False, 4000), (True, 4000), (False, 9000)])
def test_gradients_against_autograd(c1, deferred, first):
    w, g, W = c1
    count = 48
    st = warm(w, g, first)
    ix = O.NeighbourIndex(g.num_nodes, g.src, g.dst, g.ts)
    Wc = {k: v.copy() for k, v in W.items()}
    if deferred:  # a first step leaves the winners the second one applies
        T.train_step(st, g.src, g.dst, g.ts, g.edge_feat, Wc, first - count, count,
                     S.make_negatives(w, g, first - count, count), w.num_neighbors, w.num_heads, 0.0, index=ix, deferred=True)
    applied = list(st.pending) if deferred else None
    if not deferred:
        eids = np.arange(first, first + count)
        applied = []
        for u, (b, role) in O.find_winners(g.src[eids], g.dst[eids], g.ts[eids], eids).items():
            applied.append((int(u), int(g.dst[eids[b]]) if role == 0 else int(g.src[eids[b]]), int(eids[b]), float(g.ts[eids[b]])))
    before = {u: (st.mem[u].copy(), st.mem[o].copy(), float(st.last_update[u])) for u, o, _, _ in applied}
    neg = S.make_negatives(w, g, first, count)
    out, loss, grads = T.train_step(st, g.src, g.dst, g.ts, g.edge_feat, Wc, first, count, neg, w.num_neighbors,
                                    w.num_heads, 0.0, index=ix, deferred=deferred)
    Wt = {k: torch.tensor(W[k].astype(np.float64), requires_grad=True) for k in T.PARAMS}
    lt = torch_loss(Wt, w, g, applied, before, st.mem, out, count)
    assert float(lt.detach()) == pytest.approx(loss, rel=2e-6)     # (the oracle's loss is taken from float32 scores)
    lt.backward()
    for k in T.PARAMS:
        ref = Wt[k].grad.numpy()
        scale = np.abs(ref).max()
        if k == "b_K":
            # the key bias shifts every score of a head alike and cancels in the softmax: its gradient
            # is zero, and both sides leave only rounding noise
            assert scale < 1e-15 and np.abs(grads[k]).max() < 1e-15
            continue
        assert scale > 1e-9, k
        assert np.allclose(grads[k], ref, rtol=2e-5, atol=2e-6 * scale), k


def test_gradients_against_finite_differences(c1):
    w, g, W = c1
    first, count = 6000, 40
    ix = O.NeighbourIndex(g.num_nodes, g.src, g.dst, g.ts)
    neg = S.make_negatives(w, g, first, count)
    base = warm(w, g, first)
    _, _, grads = T.train_step(base.copy(), g.src, g.dst, g.ts, g.edge_feat, {k: v.copy() for k, v in W.items()}, first,
                               count, neg, w.num_neighbors, w.num_heads, 0.0, index=ix)

    def loss_at(name, idx, delta):
        Wp = {k: v.copy() for k, v in W.items()}
        Wp[name][idx] += np.float32(delta)
        st = base.copy()
        out = O.step(st, g.src, g.dst, g.ts, g.edge_feat, Wp, first, count, neg, w.num_neighbors, w.num_heads, index=ix)
        # float64 scores would be smoother; the stored float32 scores are what the step returns
        return T.bce_loss(out["score_pos"], out["score_neg"]), float(Wp[name][idx]) - float(W[name][idx])

    rng = np.random.default_rng(2)
    for name in ("w_d2", "W_d1", "W_m2", "W_m1", "W_O", "W_V", "W_K", "W_Q", "W_i", "W_h", "b_i", "time_b", "b_m1"):
        flat = np.abs(grads[name]).ravel()
        idx = np.unravel_index(int(np.argsort(flat)[-1 - int(rng.integers(0, 3))]), grads[name].shape)
        (lp, dp), (lm, dm) = loss_at(name, idx, 2e-2), loss_at(name, idx, -2e-2)
        fd = (lp - lm) / (dp - dm)
        assert fd == pytest.approx(grads[name][idx], rel=3e-2, abs=2e-5), (name, idx)


def test_sgd_update(c1):
    w, g, W = c1
    ix = O.NeighbourIndex(g.num_nodes, g.src, g.dst, g.ts)
    neg = S.make_negatives(w, g, 5000, 50)
    W0 = {k: v.copy() for k, v in W.items()}
    W1 = {k: v.copy() for k, v in W.items()}
    _, loss0, grads = T.train_step(warm(w, g, 5000), g.src, g.dst, g.ts, g.edge_feat, W0, 5000, 50, neg, w.num_neighbors,
                                   w.num_heads, 0.0, index=ix)
    _, loss1, _ = T.train_step(warm(w, g, 5000), g.src, g.dst, g.ts, g.edge_feat, W1, 5000, 50, neg, w.num_neighbors,
                               w.num_heads, 0.5, index=ix)
    assert loss1 == loss0                                  # the update comes after the loss
    for k in T.PARAMS:
        assert np.array_equal(W1[k], (W[k].astype(np.float64) - 0.5 * grads[k]).astype(np.float32))
    # a step along the negative gradient lowers the loss of the same batch
    _, loss2, _ = T.train_step(warm(w, g, 5000), g.src, g.dst, g.ts, g.edge_feat, W1, 5000, 50, neg, w.num_neighbors,
                               w.num_heads, 0.0, index=ix)
    assert loss2 < loss0


def test_relu_ties_and_inverted_gates(c1):
    # the options a float32 comparison uses where a pre-activation is within rounding of zero
    w, g, W = c1
    ix = O.NeighbourIndex(g.num_nodes, g.src, g.dst, g.ts)
    B = 40
    neg = S.make_negatives(w, g, 5000, B)

    def step(**kw):
        return T.train_step(warm(w, g, 5000), g.src, g.dst, g.ts, g.edge_feat, {k: v.copy() for k, v in W.items()}, 5000,
                            B, neg, w.num_neighbors, w.num_heads, 0.0, index=ix, **kw)
    out0, _, g0 = step()
    assert "relu_ties" not in out0
    # a huge threshold lists every unit the backward pass went through, and changes nothing else
    out1, _, g1 = step(tie_eps=1e9)
    E = w.emb_dim
    dec = [t for t in out1["relu_ties"] if t[1] == "dec"]
    merge = [t for t in out1["relu_ties"] if t[1] == "merge"]
    assert len(dec) == 2 * B * E and len(merge) % E == 0 and 0 < len(merge) <= 3 * B * E
    assert all(np.array_equal(g0[k], g1[k]) for k in T.PARAMS)
    # inverting the gate of an ACTIVE decoder unit removes exactly its term d logit * w_d2[j] from b_d1[j]
    # (pair p < B is event p against its destination: d logit = -sigmoid(-logit) / B)
    p, j = next((t[2], t[3]) for t in dec if t[2] < B and t[0] > 1e-3 and
                (W["W_d1"][t[3]].astype(np.float64) @ np.concatenate([out0["emb"][t[2]], out0["emb"][B + t[2]]]).astype(np.float64)
                 + W["b_d1"][t[3]]) > 0)
    _, _, g2 = step(relu_flip=frozenset([("dec", p, j)]))
    dlogit = -O.sigmoid(-float(out0["score_pos"][p])) / B
    assert g2["b_d1"][j] - g0["b_d1"][j] == pytest.approx(-dlogit * float(W["w_d2"][j]), rel=1e-9)
    others = np.delete(np.arange(E), j)
    assert np.array_equal(g2["b_d1"][others], g0["b_d1"][others])
    assert np.array_equal(g2["w_d2"], g0["w_d2"]) and np.array_equal(g2["b_d2"], g0["b_d2"])   # the forward is untouched
    assert not np.array_equal(g2["W_m2"], g0["W_m2"])                                          # ... what lies upstream is not
    # inverting it twice is the identity
    _, _, g3 = step(relu_flip=frozenset([("dec", p, j), ("merge", 0, 0)]))
    _, _, g4 = step(relu_flip=frozenset([("merge", 0, 0)]))
    assert g3["b_d1"][j] - g4["b_d1"][j] == pytest.approx(-dlogit * float(W["w_d2"][j]), rel=1e-9)


@pytest.mark.parametrize("H", [1, 2, 4])
def test_reassociated_attention_backward_is_the_direct_form(H):
    # The training kernels run the attention core with q~_h = W_K,h^T Qv_h (scores <q~_h, kv_k> / sqrt(d_h): the
    # key bias adds a constant over the slots, which the softmax cancels) and head output W_V,h (sum_k p_hk kv_k)
    # + b_V,h, forward and backward.  In exact arithmetic that is the direct form the oracle differentiates:
    # every gradient below is formed both ways in float64.
    rng = np.random.default_rng(7 + H)
    c, d_a, d_kv = 7, 8 * H, 11
    d_h = d_a // H
    Qv, kv = rng.normal(size=d_a), rng.normal(size=(c, d_kv))
    W_K, W_V = rng.normal(size=(d_a, d_kv)), rng.normal(size=(d_a, d_kv))
    b_K, b_V = rng.normal(size=d_a), rng.normal(size=d_a)
    do = rng.normal(size=d_a)                      # gradient of the heads' outputs
    # ---- direct form (the oracle's statements)
    Kp, Vp = kv @ W_K.T + b_K, kv @ W_V.T + b_V
    o = np.zeros(d_a)
    dQv, dKp, dVp = np.zeros(d_a), np.zeros_like(Kp), np.zeros_like(Vp)
    probs = []
    for h in range(H):
        sl = slice(h * d_h, (h + 1) * d_h)
        s = Kp[:, sl] @ Qv[sl] / np.sqrt(d_h)
        a = np.exp(s - s.max())
        a /= a.sum()
        probs.append(a)
        o[sl] = a @ Vp[:, sl]
        dVp[:, sl] = np.outer(a, do[sl])
        da = Vp[:, sl] @ do[sl]
        ds = a * (da - a @ da)
        dQv[sl] = ds @ Kp[:, sl] / np.sqrt(d_h)
        dKp[:, sl] = np.outer(ds, Qv[sl]) / np.sqrt(d_h)
    dW_K, db_K, dW_V, db_V = dKp.T @ kv, dKp.sum(axis=0), dVp.T @ kv, dVp.sum(axis=0)
    dkv = dKp @ W_K + dVp @ W_V
    # ---- re-associated form (what the kernels compute: products over the query, vectors over the slots)
    o2, dQv2, dkv2 = np.zeros(d_a), np.zeros(d_a), np.zeros_like(kv)
    dW_K2, dW_V2, db_V2 = np.zeros_like(W_K), np.zeros_like(W_V), np.zeros(d_a)
    for h in range(H):
        sl = slice(h * d_h, (h + 1) * d_h)
        qt = W_K[sl].T @ Qv[sl]                              # q~_h
        s = kv @ qt / np.sqrt(d_h)                           # scores up to the constant <b_K,h, Qv_h> / sqrt(d_h)
        a = np.exp(s - s.max())
        a /= a.sum()
        assert np.allclose(a, probs[h], rtol=1e-12, atol=1e-15)
        kvb = a @ kv                                         # sum_k p_hk kv_k
        o2[sl] = W_V[sl] @ kvb + b_V[sl]
        dkvb = W_V[sl].T @ do[sl]                            # d(sum_k p_hk kv_k)
        dW_V2[sl] = np.outer(do[sl], kvb)
        db_V2[sl] = do[sl]
        dp = kv @ dkvb
        ds = a * (dp - a @ dp) / np.sqrt(d_h)                # gradient of <q~_h, kv_k>
        dqt = ds @ kv
        dkv2 += np.outer(a, dkvb) + np.outer(ds, qt)
        dQv2[sl] = W_K[sl] @ dqt
        dW_K2[sl] = np.outer(Qv[sl], dqt)
    for got, want in ((o2, o), (dQv2, dQv), (dkv2, dkv), (dW_K2, dW_K), (dW_V2, dW_V), (db_V2, db_V)):
        assert np.allclose(got, want, rtol=1e-10, atol=1e-12)
    assert np.abs(db_K).max() < 1e-12                        # softmax shift invariance: the key bias takes no gradient
