"""Pins for the oracle's building blocks: each is checked against something other than
itself -- hand-derived closed forms (tests/golden), library routines in float64, invariants."""
import json
import math
import os

import numpy as np
import pytest
import torch

from oracle import tig_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
_NS = {"ln2": math.log(2.0), "ln3": math.log(3.0)}


def _ev(x):
    if isinstance(x, list):
        return np.array([_ev(v) for v in x], dtype=np.float64)
    return float(eval(x, {"__builtins__": {}}, _NS))


def _rand_weights(rng, M, T, F, E):
    import tig_synth
    shapes = tig_synth.weight_shapes(M, T, F, E)
    return {k: rng.uniform(-0.5, 0.5, size=s).astype(np.float32) for k, s in shapes.items()}


# ----------------------------------------------------------------------------- time encoding


def test_time_encode_zero_is_cos_b():
    b = np.array([0.0, 0.5, -1.0], dtype=np.float32)
    w = np.array([1.0, 0.1, 3.0], dtype=np.float32)
    out = O.time_encode(0.0, w, b)
    assert out.dtype == np.float32
    np.testing.assert_array_equal(out, np.cos(b.astype(np.float64)).astype(np.float32))
    assert O.time_encode(0.0, w, np.zeros(3, np.float32)).tolist() == [1.0, 1.0, 1.0]


def test_time_encode_full_periods():
    # w = 1/8 is exact in binary, so w * x = 2*pi*n up to the rounding of x itself
    w = np.array([0.125], dtype=np.float32)
    b = np.array([0.0], dtype=np.float32)
    for n in (1, 7, 40000):
        x = 2.0 * math.pi * n / 0.125
        assert abs(float(O.time_encode(x, w, b)[0]) - 1.0) < 1e-6


def test_time_encode_against_extended_precision():
    rng = np.random.default_rng(1)
    w = (10.0 ** rng.uniform(-9, 0, size=64)).astype(np.float32)
    b = rng.uniform(-math.pi, math.pi, size=64).astype(np.float32)
    xs = np.concatenate([rng.uniform(0, 2.6e6, size=50), [2.6e6, 0.0, 1.0]])
    got = O.time_encode(xs, w, b).astype(np.float64)
    ld = np.longdouble
    want = np.cos(xs.astype(ld)[:, None] * w.astype(ld) + b.astype(ld)).astype(np.float64)
    # float32 storage: half an ulp near 1 is 6e-8; float64 argument error at 2.6e6 is ~5e-10
    assert np.max(np.abs(got - want)) < 7e-8
    assert got.shape == (53, 64)


# ----------------------------------------------------------------------------- GRU


def test_gru_hand_example():
    g = json.load(open(os.path.join(GOLDEN, "gru_hand_2d.json")))
    out = O.gru_cell(_ev(g["m"]), _ev(g["h"]), _ev(g["W_i"]), _ev(g["b_i"]), _ev(g["W_h"]),
                     _ev(g["b_h"]))
    np.testing.assert_allclose(out, _ev(g["h_new"]), rtol=0, atol=1e-14)


def test_gru_closed_forms():
    rng = np.random.default_rng(2)
    M, D = 5, 9
    h = rng.normal(size=M)
    m = rng.normal(size=D)
    Z = np.zeros
    # all parameters zero: r = z = 1/2, n = 0  =>  h' = h / 2
    np.testing.assert_allclose(O.gru_cell(m, h, Z((3 * M, D)), Z(3 * M), Z((3 * M, M)), Z(3 * M)),
                               0.5 * h, atol=1e-15)
    # update gate saturated at 1: h' = h
    W_i, W_h = rng.normal(size=(3 * M, D)), rng.normal(size=(3 * M, M))
    b_i, b_h = rng.normal(size=3 * M), rng.normal(size=3 * M)
    b_i2 = b_i.copy()
    b_i2[M:2 * M] = 400.0
    np.testing.assert_allclose(O.gru_cell(m, h, W_i, b_i2, W_h, b_h), h, atol=1e-12)
    # update gate saturated at 0 and no input/hidden weights on n:
    # h' = tanh(b_in + sig(r_pre) * b_hn)
    W_i3, W_h3 = W_i.copy(), W_h.copy()
    W_i3[2 * M:] = 0.0
    W_h3[2 * M:] = 0.0
    b_i3 = b_i.copy()
    b_i3[M:2 * M] = -400.0
    r = 1.0 / (1.0 + np.exp(-(W_i[:M] @ m + b_i[:M] + W_h[:M] @ h + b_h[:M])))
    np.testing.assert_allclose(O.gru_cell(m, h, W_i3, b_i3, W_h3, b_h),
                               np.tanh(b_i[2 * M:] + r * b_h[2 * M:]), atol=1e-12)


def test_gru_equals_library_cell():
    rng = np.random.default_rng(3)
    M, D = 12, 31
    cell = torch.nn.GRUCell(D, M, bias=True, dtype=torch.float64)
    W_i = cell.weight_ih.detach().numpy()
    W_h = cell.weight_hh.detach().numpy()
    b_i = cell.bias_ih.detach().numpy()
    b_h = cell.bias_hh.detach().numpy()
    for _ in range(5):
        m, h = rng.normal(size=D), rng.normal(size=M)
        want = cell(torch.from_numpy(m)[None], torch.from_numpy(h)[None])[0].detach().numpy()
        np.testing.assert_allclose(O.gru_cell(m, h, W_i, b_i, W_h, b_h), want, atol=1e-13)


# ----------------------------------------------------------------------------- attention


def test_attention_hand_example():
    g = json.load(open(os.path.join(GOLDEN, "attention_hand.json")))
    W = {k: _ev(g[k]) for k in ("W_Q", "b_Q", "W_K", "b_K", "W_V", "b_V", "W_O", "b_O")}
    out = O.attention(_ev(g["q_in"]), _ev(g["kv"]), W, g["H"])
    np.testing.assert_allclose(out, _ev(g["attn"]), rtol=0, atol=1e-14)


def _attn_weights(rng, d_a, d_kv):
    return {"W_Q": rng.normal(size=(d_a, d_a)), "b_Q": rng.normal(size=d_a),
            "W_K": rng.normal(size=(d_a, d_kv)), "b_K": rng.normal(size=d_a),
            "W_V": rng.normal(size=(d_a, d_kv)), "b_V": rng.normal(size=d_a),
            "W_O": rng.normal(size=(d_a, d_a)), "b_O": rng.normal(size=d_a)}


def test_attention_special_cases():
    rng = np.random.default_rng(4)
    d_a, d_kv, H = 8, 11, 2
    W = _attn_weights(rng, d_a, d_kv)
    q = rng.normal(size=d_a)
    kv = rng.normal(size=(6, d_kv))
    # empty neighbourhood: zero vector (no bias)
    assert np.all(O.attention(q, kv[:0], W, H) == 0.0)
    # one neighbour: weight 1, attn = W_O (W_V kv + b_V) + b_O
    np.testing.assert_allclose(O.attention(q, kv[:1], W, H),
                               W["W_O"] @ (W["W_V"] @ kv[0] + W["b_V"]) + W["b_O"], atol=1e-12)
    # zero query projection: uniform weights, o = mean of the value rows
    W0 = dict(W, W_Q=np.zeros((d_a, d_a)), b_Q=np.zeros(d_a))
    vmean = (kv @ W["W_V"].T + W["b_V"]).mean(axis=0)
    np.testing.assert_allclose(O.attention(q, kv, W0, H), W["W_O"] @ vmean + W["b_O"], atol=1e-12)
    # identical rows: independent of how many
    rep = np.repeat(kv[:1], 5, axis=0)
    np.testing.assert_allclose(O.attention(q, rep, W, H), O.attention(q, kv[:1], W, H), atol=1e-12)
    # permutation of the neighbour slots
    perm = rng.permutation(6)
    np.testing.assert_allclose(O.attention(q, kv[perm], W, H), O.attention(q, kv, W, H), atol=1e-12)
    # the key bias is constant over the slots and cancels in the softmax
    Wb = dict(W, b_K=W["b_K"] + 3.0)
    np.testing.assert_allclose(O.attention(q, kv, Wb, H), O.attention(q, kv, W, H), atol=1e-11)


@pytest.mark.parametrize("H", [1, 2, 4])
def test_attention_equals_library_multihead(H):
    rng = np.random.default_rng(5)
    d_a, d_kv, cnt = 8, 13, 7
    W = _attn_weights(rng, d_a, d_kv)
    q = rng.normal(size=d_a)
    kv = rng.normal(size=(cnt, d_kv))
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a))
    pad = 3  # padded key slots masked out, like the unused neighbour slots
    kv_pad = np.concatenate([kv, rng.normal(size=(pad, d_kv))])
    mask = torch.zeros(1, cnt + pad, dtype=torch.bool)
    mask[0, cnt:] = True
    out, _ = torch.nn.functional.multi_head_attention_forward(
        query=t(q)[None, None, :], key=t(kv_pad)[:, None, :], value=t(kv_pad)[:, None, :],
        embed_dim_to_check=d_a, num_heads=H, in_proj_weight=None,
        in_proj_bias=t(np.concatenate([W["b_Q"], W["b_K"], W["b_V"]])),
        bias_k=None, bias_v=None, add_zero_attn=False, dropout_p=0.0,
        out_proj_weight=t(W["W_O"]), out_proj_bias=t(W["b_O"]), training=False,
        key_padding_mask=mask, need_weights=False, use_separate_proj_weight=True,
        q_proj_weight=t(W["W_Q"]), k_proj_weight=t(W["W_K"]), v_proj_weight=t(W["W_V"]))
    np.testing.assert_allclose(O.attention(q, kv, W, H), out[0, 0].numpy(), atol=1e-12)


# ----------------------------------------------------------------------------- merge / decoder


def test_merge_and_decoder_selectors():
    d_a, M, E = 4, 3, 3
    attn = np.array([0.5, -2.0, 3.0, 1.0])
    mem_u = np.array([7.0, -1.0, 2.0])
    W = {"W_m1": np.zeros((E, d_a + M)), "b_m1": np.zeros(E), "W_m2": np.eye(E), "b_m2": np.zeros(E),
         "W_d1": np.zeros((E, 2 * E)), "b_d1": np.zeros(E), "w_d2": np.ones(E), "b_d2": np.array([0.25])}
    W["W_m1"][0, 0] = 1.0      # attn[0] = 0.5   -> passes the ReLU
    W["W_m1"][1, 1] = 1.0      # attn[1] = -2    -> clipped to 0
    W["W_m1"][2, d_a] = 1.0    # mem_u[0] = 7    -> shows the [attn | s_u] order
    np.testing.assert_allclose(O.merge(attn, mem_u, W), [0.5, 0.0, 7.0])
    W["b_m2"] = np.array([1.0, 1.0, 1.0])
    np.testing.assert_allclose(O.merge(attn, mem_u, W), [1.5, 1.0, 8.0])
    a, b = np.array([1.0, 2.0, 3.0]), np.array([10.0, -20.0, 30.0])
    W["W_d1"][0, 1] = 1.0          # a[1] = 2
    W["W_d1"][1, E + 1] = 1.0      # b[1] = -20 -> clipped
    W["W_d1"][2, E + 2] = 0.5      # b[2] / 2 = 15
    assert O.decoder(a, b, W) == pytest.approx(2.0 + 0.0 + 15.0 + 0.25)
    assert O.decoder(b, a, W) == pytest.approx(0.0 + 2.0 + 1.5 + 0.25)


def test_merge_decoder_against_float64_matmul():
    rng = np.random.default_rng(6)
    W = _rand_weights(rng, 6, 4, 3, 5)
    attn, mem_u = rng.normal(size=10), rng.normal(size=6).astype(np.float32)
    x = torch.from_numpy(np.concatenate([attn, mem_u.astype(np.float64)]))
    tw = {k: torch.from_numpy(v.astype(np.float64)) for k, v in W.items()}
    want = torch.nn.functional.linear(torch.relu(torch.nn.functional.linear(x, tw["W_m1"], tw["b_m1"])),
                                      tw["W_m2"], tw["b_m2"]).numpy()
    np.testing.assert_allclose(O.merge(attn, mem_u, W), want, atol=1e-13)
    ea, eb = rng.normal(size=5), rng.normal(size=5)
    xx = torch.from_numpy(np.concatenate([ea, eb]))
    want = float(tw["w_d2"] @ torch.relu(torch.nn.functional.linear(xx, tw["W_d1"], tw["b_d1"])) + tw["b_d2"][0])
    assert O.decoder(ea, eb, W) == pytest.approx(want, abs=1e-13)


def test_decoder_layer_one_folded_through_merge_layer_two():
    """Decoder layer 1 applied to the merge hidden layer h1 through W_d1a W_m2, W_d1b W_m2 and
    b_d1 + (W_d1a + W_d1b) b_m2 (the form one phase of the embedding kernel computes) is the
    decoder of the two embeddings."""
    rng = np.random.default_rng(16)
    M, T, F, E = 6, 4, 3, 5
    W = _rand_weights(rng, M, T, F, E)
    f64 = np.float64
    Wm2, bm2 = W["W_m2"].astype(f64), W["b_m2"].astype(f64)
    Wa, Wb = W["W_d1"].astype(f64)[:, :E], W["W_d1"].astype(f64)[:, E:]
    bias = W["b_d1"].astype(f64) + (Wa + Wb) @ bm2
    for _ in range(5):
        rows = []
        for _ in range(2):
            attn, mem_u = rng.normal(size=M + T), rng.normal(size=M).astype(np.float32)
            h1 = np.maximum(W["W_m1"].astype(f64) @ np.concatenate([attn, mem_u.astype(f64)])
                            + W["b_m1"].astype(f64), 0.0)
            rows.append((O.merge(attn, mem_u, W), h1))
        (emb_a, h1_a), (emb_b, h1_b) = rows
        folded = W["w_d2"].astype(f64) @ np.maximum((Wa @ Wm2) @ h1_a + (Wb @ Wm2) @ h1_b + bias, 0.0) \
            + W["b_d2"].astype(f64)[0]
        assert O.decoder(emb_a, emb_b, W) == pytest.approx(float(folded), abs=1e-12)


# ----------------------------------------------------------------------------- winners


def test_winners_hand_cases():
    #            b:  0  1  2  3  4
    src = np.array([5, 1, 5, 2, 9])
    dst = np.array([1, 2, 3, 5, 5])
    ts = np.array([1.0, 1.0, 2.0, 2.0, 2.0])
    eid = np.arange(100, 105)
    w = O.find_winners(src, dst, ts, eid)
    # node 5 occurs in events 0, 2 (src) and 3, 4 (dst); its last is b = 4 as destination
    assert w == {5: (4, 1), 1: (1, 0), 2: (3, 0), 3: (2, 1), 9: (4, 0)}


def test_winners_equal_last_occurrence_reverse_scan():
    rng = np.random.default_rng(7)
    for _ in range(20):
        B = 50
        src = rng.integers(0, 12, size=B)
        dst = (src + rng.integers(1, 12, size=B)) % 12
        ts = np.sort(rng.integers(0, 10, size=B)).astype(np.float64)
        eid = np.arange(1000, 1000 + B)
        want = {}
        for b in range(B - 1, -1, -1):      # sorted stream: last occurrence wins
            want.setdefault(int(dst[b]), (b, 1))
            want.setdefault(int(src[b]), (b, 0))
        got = O.find_winners(src, dst, ts, eid)
        # src and dst of one event are different nodes, so the setdefault order within an
        # event does not matter
        assert got == want


def test_winners_use_time_then_event_id():
    # deliberately NOT sorted by time: the key is (time, event id), not the position
    src = np.array([1, 1, 1])
    dst = np.array([2, 3, 4])
    ts = np.array([5.0, 9.0, 9.0])
    eid = np.array([12, 10, 11])
    w = O.find_winners(src, dst, ts, eid)
    assert w[1] == (2, 0)           # time 9.0 twice -> greater event id 11 (position 2)
    eid2 = np.array([12, 11, 10])
    assert O.find_winners(src, dst, ts, eid2)[1] == (1, 0)
