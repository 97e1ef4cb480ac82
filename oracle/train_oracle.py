"""CPU oracle of one TRAINING step of the TIG model.  TEST INFRASTRUCTURE ONLY.

The batch step of oracle/tig_oracle.py followed by the self-supervised signal of the paper's
Sec. II-C (the decoder's edge probabilities of the batch's events against one sampled negative
each) and "Backward and Optimize" of Alg. 2: binary cross-entropy on the logits, the gradient of
every weight by hand-written reverse-mode differentiation in float64, and a plain SGD update.
Imported only by tests and the benchmark's CPU-baseline leg; shares no code with the library.

Readings where the paper is silent (it names neither the loss nor the optimiser):
  * loss = mean_b softplus(-logit_pos[b]) + mean_b softplus(logit_neg[b])  (binary cross-entropy
    with logits, positives labelled 1 and negatives 0, each averaged over the batch);
  * the node memory is a constant of the step: gradients flow into the GRU only through the rows
    the step itself overwrites (the embedding reads them), never into rows stored by earlier
    steps, and not into edge features; within the step a message's inputs (the memory at the
    start of the step) are constants as well;
  * values the method stores in float32 (messages, memory rows, key/value rows, embeddings,
    scores) are differentiated as if the rounding were the identity;
  * relu'(0) = 0 (a float32 implementation can land on the other side of zero where a pre-activation
    is within its rounding error of zero: `tie_eps` reports such units, `relu_flip` evaluates the
    gradients with the gate of listed units inverted, so that a comparison can accept either side);
  * optimiser: W <- W - lr * dL/dW in float32 (SGD without momentum).

Pins (tests/test_oracle_train.py): the forward equals tig_oracle.step bit for bit; every gradient
against float64 torch.autograd of an independently written forward, and against central finite
differences of the loss; loss closed forms; an SGD step with lr = 0 changes nothing.
"""
from __future__ import annotations

import numpy as np

from . import tig_oracle as O

f32, f64 = np.float32, np.float64

PARAMS = ("time_w", "time_b", "W_i", "b_i", "W_h", "b_h", "W_Q", "b_Q", "W_K", "b_K", "W_V", "b_V", "W_O", "b_O",
          "W_m1", "b_m1", "W_m2", "b_m2", "W_d1", "b_d1", "w_d2", "b_d2")


def softplus(x):
    return np.logaddexp(0.0, x)


def bce_loss(score_pos, score_neg):
    return float(np.mean(softplus(-score_pos.astype(f64))) + np.mean(softplus(score_neg.astype(f64))))


def train_step(state, src, dst, ts, edge_feat, W, first_eid, count, neg_dst, K, H, lr, index=None,
               deferred=False, tie_eps=0.0, relu_flip=frozenset()):
    """One training step.  Runs tig_oracle.step (state updated in place), then loss, gradients and
    the SGD update of W (in place).  Returns (the step's outputs, loss, grads: dict name -> float64).
    tie_eps > 0: the outputs carry "relu_ties", the ReLU units whose pre-activation is closer to zero
    than tie_eps, as (|pre-activation|, layer, row, unit) with layer "dec" (row = pair index: event b
    against its destination, count + b against its negative) or "merge" (row = query index).
    relu_flip: units (layer, row, unit) whose gate is taken as the opposite of (pre-activation > 0)."""
    M = state.mem.shape[1]
    T = W["time_w"].shape[0]
    F = edge_feat.shape[1]
    # what the GRU of this step reads: the rows of the applied batch's winners, before the overwrite
    eids = np.arange(first_eid, first_eid + count)
    if deferred:
        applied = list(state.pending)
    else:
        applied = []
        for u, (b, role) in O.find_winners(src[eids], dst[eids], ts[eids], eids).items():
            other = int(dst[eids[b]]) if role == 0 else int(src[eids[b]])
            applied.append((int(u), other, int(eids[b]), float(ts[eids[b]])))
    before = {u: (state.mem[u].copy(), state.mem[o].copy(), float(state.last_update[u])) for u, o, _, _ in applied}

    out = O.step(state, src, dst, ts, edge_feat, W, first_eid, count, neg_dst, K, H, index=index, deferred=deferred)
    loss = bce_loss(out["score_pos"], out["score_neg"])

    Wd = {k: W[k].astype(f64) for k in PARAMS}
    g = {k: np.zeros_like(Wd[k]) for k in PARAMS}
    E = Wd["W_m2"].shape[0]
    d_a = Wd["W_Q"].shape[0]
    d_h = d_a // H
    emb = out["emb"].astype(f64)
    B = count

    # ---- decoder: d loss / d logit, back to the embeddings
    d_emb = np.zeros_like(emb)
    pairs = [(b, B + b, out["score_pos"][b], -1.0) for b in range(B)] + \
            [(b, 2 * B + b, out["score_neg"][b], +1.0) for b in range(B)]
    ties = []
    flips = {}
    for layer, row, unit in relu_flip:
        flips.setdefault((layer, int(row)), []).append(int(unit))

    def relu_gate(pre, layer, row):
        gate = pre > 0.0
        if tie_eps > 0.0:
            for j in np.nonzero(np.abs(pre) < tie_eps)[0]:
                ties.append((float(abs(pre[j])), layer, row, int(j)))
        for j in flips.get((layer, row), ()):
            gate[j] = not gate[j]
        return gate

    for p_idx, (qa, qb, logit, sign) in enumerate(pairs):
        # d softplus(sign * logit) / d logit = sign * sigmoid(sign * logit), averaged over the batch
        dlogit = sign * O.sigmoid(sign * float(logit)) / B
        x = np.concatenate([emb[qa], emb[qb]])
        y = Wd["W_d1"] @ x + Wd["b_d1"]
        hid = np.maximum(y, 0.0)
        g["w_d2"] += dlogit * hid
        g["b_d2"] += dlogit
        dy = dlogit * Wd["w_d2"] * relu_gate(y, "dec", p_idx)
        g["W_d1"] += np.outer(dy, x)
        g["b_d1"] += dy
        dx = Wd["W_d1"].T @ dy
        d_emb[qa] += dx[:E]
        d_emb[qb] += dx[E:]

    # ---- embedding of every query: merge MLP and attention, back to the state rows it read
    updated = {u for u, _, _, _ in applied}
    d_mem = {u: np.zeros(M, dtype=f64) for u in updated}   # gradient w.r.t. the rows this step wrote
    phi0 = O.time_encode(0.0, W["time_w"], W["time_b"]).astype(f64)
    tw, tb = Wd["time_w"], Wd["time_b"]
    q_node, q_time = out["q_node"], out["q_time"]
    for q in range(emb.shape[0]):
        if not d_emb[q].any():
            continue
        u = int(q_node[q])
        c = int(out["nbr_cnt"][q])
        s_u = state.mem[u].astype(f64)
        q_in = np.concatenate([s_u, phi0])
        if c > 0:
            vs = out["nbr_node"][q, :c]
            dts = q_time[q] - out["nbr_ts"][q, :c]
            phi_k = O.time_encode(dts, W["time_w"], W["time_b"])
            kv = np.concatenate([state.mem[vs], edge_feat[out["nbr_eid"][q, :c]], phi_k], axis=1).astype(f32).astype(f64)
            Qv = Wd["W_Q"] @ q_in + Wd["b_Q"]
            Kp = kv @ Wd["W_K"].T + Wd["b_K"]
            Vp = kv @ Wd["W_V"].T + Wd["b_V"]
            o = np.zeros(d_a)
            probs = []
            for h in range(H):
                sl = slice(h * d_h, (h + 1) * d_h)
                s = Kp[:, sl] @ Qv[sl] / np.sqrt(float(d_h))
                a = np.exp(s - s.max())
                a /= a.sum()
                probs.append(a)
                o[sl] = a @ Vp[:, sl]
            attn = Wd["W_O"] @ o + Wd["b_O"]
        else:
            attn = np.zeros(d_a)
        x = np.concatenate([attn, s_u])
        z1 = Wd["W_m1"] @ x + Wd["b_m1"]
        h1 = np.maximum(z1, 0.0)
        # backward
        de = d_emb[q]
        g["W_m2"] += np.outer(de, h1)
        g["b_m2"] += de
        dz1 = (Wd["W_m2"].T @ de) * relu_gate(z1, "merge", q)
        g["W_m1"] += np.outer(dz1, x)
        g["b_m1"] += dz1
        dx = Wd["W_m1"].T @ dz1
        d_attn, ds_u = dx[:d_a], dx[d_a:].copy()
        if c > 0:
            g["W_O"] += np.outer(d_attn, o)
            g["b_O"] += d_attn
            do = Wd["W_O"].T @ d_attn
            dQv = np.zeros(d_a)
            dKp = np.zeros_like(Kp)
            dVp = np.zeros_like(Vp)
            for h in range(H):
                sl = slice(h * d_h, (h + 1) * d_h)
                a = probs[h]
                dVp[:, sl] = np.outer(a, do[sl])
                da = Vp[:, sl] @ do[sl]
                ds = a * (da - a @ da)
                dQv[sl] = ds @ Kp[:, sl] / np.sqrt(float(d_h))
                dKp[:, sl] = np.outer(ds, Qv[sl]) / np.sqrt(float(d_h))
            g["W_Q"] += np.outer(dQv, q_in)
            g["b_Q"] += dQv
            dq_in = Wd["W_Q"].T @ dQv
            ds_u += dq_in[:M]
            g["time_b"] += -np.sin(tb) * dq_in[M:]           # Phi(0) = cos(b)
            g["W_K"] += dKp.T @ kv
            g["b_K"] += dKp.sum(axis=0)
            g["W_V"] += dVp.T @ kv
            g["b_V"] += dVp.sum(axis=0)
            dkv = dKp @ Wd["W_K"] + dVp @ Wd["W_V"]
            for k in range(c):
                v = int(vs[k])
                if v in updated:
                    d_mem[v] += dkv[k, :M]
                sin_k = np.sin(tw * dts[k] + tb)
                dphi = dkv[k, M + F:]
                g["time_w"] += -sin_k * dts[k] * dphi
                g["time_b"] += -sin_k * dphi
        if u in updated:
            d_mem[u] += ds_u

    # ---- GRU and message of the applied winners
    for u, other, eid, t in applied:
        dh = d_mem[u]
        if not dh.any():
            continue
        mem_u, mem_o, lu_u = before[u]
        dt = t - lu_u
        phi = O.time_encode(dt, W["time_w"], W["time_b"])
        m = np.concatenate([mem_u, mem_o, phi, edge_feat[eid]]).astype(f32).astype(f64)
        h = mem_u.astype(f64)
        gi = Wd["W_i"] @ m + Wd["b_i"]
        gh = Wd["W_h"] @ h + Wd["b_h"]
        r = O.sigmoid(gi[:M] + gh[:M])
        z = O.sigmoid(gi[M:2 * M] + gh[M:2 * M])
        n = np.tanh(gi[2 * M:] + r * gh[2 * M:])
        dn = dh * (1.0 - z)
        dz = dh * (h - n)
        dpre_n = dn * (1.0 - n * n)
        dr = dpre_n * gh[2 * M:]
        dpre_r = dr * r * (1.0 - r)
        dpre_z = dz * z * (1.0 - z)
        dgi = np.concatenate([dpre_r, dpre_z, dpre_n])
        dgh = np.concatenate([dpre_r, dpre_z, dpre_n * r])
        g["W_i"] += np.outer(dgi, m)
        g["b_i"] += dgi
        g["W_h"] += np.outer(dgh, h)
        g["b_h"] += dgh
        dm = Wd["W_i"].T @ dgi
        dphi = dm[2 * M:2 * M + T]
        sin_m = np.sin(tw * dt + tb)
        g["time_w"] += -sin_m * dt * dphi
        g["time_b"] += -sin_m * dphi

    if lr != 0.0:
        for k in PARAMS:
            W[k] = (W[k].astype(f64) - lr * g[k]).astype(f32)
    if tie_eps > 0.0:
        out["relu_ties"] = ties
    return out, loss, g
