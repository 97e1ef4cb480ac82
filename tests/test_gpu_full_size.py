"""Parity at the benchmark's full size (the one-GPU partition workload, 250 M events, batch 4000)
in the launch configuration bench.py times: whole steps against the oracle (with its indexed
neighbour routine), plus sampled queries against the brute-force definition and properties that
hold at any size."""
import numpy as np
import pytest

import tig_synth as S
from oracle import tig_oracle as O
from tests.parity import compare_step, gate
from tests.test_gpu_parity import Bundle, make_ctx, run, window, TOL

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]


@pytest.fixture(scope="module")
def c5():
    print("[c5] generating 250 M events ...", flush=True)
    b = Bundle(S.WORKLOADS["c5_gpu_partition"])
    print("[c5] generated", flush=True)
    return b


@pytest.fixture(scope="module")
def c5_ctx(c5):
    ctxs = {}

    def get(precision):
        if precision == "close":        # make room for a context of another kind
            for c in ctxs.values():
                c.close()
            ctxs.clear()
            return None
        if precision not in ctxs:
            for c in ctxs.values():     # one 30 GB context at a time
                c.close()
            ctxs.clear()
            print(f"[c5] tig_init {precision} ...", flush=True)
            ctxs[precision] = make_ctx(c5.w, c5.g, c5.W, precision)
            print("[c5] tig_init done", flush=True)
        return ctxs[precision]
    yield get
    for c in ctxs.values():
        c.close()


@pytest.mark.parametrize("precision", ["bf16", "fp32"])
def test_c5_steps_match_oracle(c5, c5_ctx, precision):
    # the launch configuration bench.py times: from the second step on two launches, the batch's
    # winners, distinct queries and GRU rows prepared by the step before
    first, bs = window(c5.w, 0.5, 3)
    run(c5, precision, bs, locked=False, warm_at=first, ctx=c5_ctx(precision), expect_launches=2)
    first, bs = window(c5.w, 0.7, 2)
    run(c5, precision, bs, locked=False, warm_at=first, ctx=c5_ctx(precision), expect_launches=2)


def test_c5_deferred_order(c5, c5_ctx):
    c5_ctx("close")
    ctx = make_ctx(c5.w, c5.g, c5.W, "bf16", order="deferred")
    first, bs = window(c5.w, 0.3, 3)
    run(c5, "bf16", bs, locked=False, warm_at=first, ctx=ctx, order="deferred", expect_launches=2)
    ctx.close()


def test_c5_sampled_queries_against_bruteforce_definition(c5, c5_ctx):
    import torch
    w, g = c5.w, c5.g
    ctx = c5_ctx("fp32")
    first, count = int(w.num_events * 0.9) // w.batch_size * w.batch_size, w.batch_size
    neg = S.make_negatives(w, g, first, count)
    out = ctx.alloc_outputs(count, with_neg=True, inspect=True)
    ctx.step(first, count, torch.from_numpy(neg).to("cuda:0"), out)
    torch.cuda.synchronize()
    nb_node, nb_eid = out.nbr_node.cpu().numpy(), out.nbr_eid.cpu().numpy()
    nb_ts, nb_cnt = out.nbr_ts.cpu().numpy(), out.nbr_cnt.cpu().numpy()
    q_node = np.concatenate([g.src[first:first + count], g.dst[first:first + count], neg])
    q_time = np.tile(g.ts[first:first + count], 3)
    # properties at full size: no future leakage, ordering, every slot is a real incident event
    valid = nb_eid >= 0
    assert np.array_equal(valid.sum(axis=1), nb_cnt)
    assert np.all(nb_ts[valid] < np.repeat(q_time, w.num_neighbors).reshape(valid.shape)[valid])
    e = nb_eid[valid]
    qn = np.repeat(q_node, w.num_neighbors).reshape(valid.shape)[valid]
    other = nb_node[valid]
    assert np.all(((g.src[e] == qn) & (g.dst[e] == other)) | ((g.dst[e] == qn) & (g.src[e] == other)))
    assert np.array_equal(nb_ts[valid], g.ts[e])
    for q in range(0, 3 * count, 997):
        c = nb_cnt[q]
        keys = list(zip(nb_ts[q, :c], nb_eid[q, :c]))
        assert keys == sorted(keys, reverse=True)
    # sampled queries against the definition (a scan of all 250 M events each)
    rng = np.random.default_rng(5)
    sample = np.concatenate([rng.integers(0, 2 * count, size=6), rng.integers(2 * count, 3 * count, size=2)])
    for q in sample:
        print(f"[c5] brute-force query {q}: node {q_node[q]} t {q_time[q]}", flush=True)
        bn, be, bt, bc = O.neighbours_bruteforce(g.src, g.dst, g.ts, int(q_node[q]), float(q_time[q]),
                                                 w.num_neighbors)
        assert bc == nb_cnt[q]
        assert np.array_equal(bn, nb_node[q]) and np.array_equal(be, nb_eid[q]) and np.array_equal(bt, nb_ts[q])


def test_c5_training_steps(c5, c5_ctx):
    # the training step at the benchmark's size: loss, every gradient, state and outputs of two
    # consecutive 4000-event batches (deferred order, as bench.py --train runs it)
    from tests.test_gpu_train import run_training
    c5_ctx("close")
    first, bs = window(c5.w, 0.5, 2)
    run_training(c5, bs, 0.0, "deferred", warm_at=first)
