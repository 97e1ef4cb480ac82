"""GPU path vs CPU oracle, through the C ABI, on the seeded synthetic workloads.

Bar: neighbour tables and last-message winners bit-exact; fp32 embeddings, memory and scores
within 1e-4, the bf16 matrix-core variant within 2e-2, both under the per-tensor gate
|got - ref| <= tol * (|ref| + mean|ref|)."""
import numpy as np
import pytest

import tig_synth as S
from oracle import tig_oracle as O
from tests.parity import compare_step, gate

pytestmark = pytest.mark.gpu

TOL = {"fp32": 1e-4, "bf16": 2e-2}


def make_ctx(w, g, W, precision, max_batch=None, order="update_first"):
    import torch
    from paper_2308_14129_amd import tig
    assert torch.cuda.is_available()
    cfg = tig.make_config(w.mem_dim, w.time_dim, w.feat_dim, w.emb_dim, w.num_neighbors, w.num_heads,
                          max_batch or w.batch_size, precision, order)
    return tig.TigContext(cfg, g.num_nodes, g.src, g.dst, g.ts, g.edge_feat, W, device="cuda:0")


class Bundle:
    """Graph + weights + oracle index of one workload, built once per module."""

    def __init__(self, w):
        self.w = w
        self.g = S.make_graph(w)
        self.W = S.make_weights(w)
        self.ix = O.NeighbourIndex(self.g.num_nodes, self.g.src, self.g.dst, self.g.ts)


def run(bundle, precision, batches, locked, warm_at=None, with_neg=True, ctx=None, order="update_first",
        expect_launches=None, quiet=False):
    """Runs the batches on both sides.  locked=True loads the oracle's state into the GPU before
    every step (step-locked parity); otherwise both sides run freely from the same start, which
    is the state after a reset or, with warm_at, the seeded warm state of a mid-stream window.
    Every step asks for the neighbour tables and the per-entry winner flags (they do not change
    what is launched) and checks that rows outside the applied batch stay bit-identical.
    order="deferred": both sides apply the previous step's winners before embedding (a state
    import drops what is kept, on both sides).
    expect_launches: kernels per step, checked from the second step on."""
    import torch
    w, g, W, ix = bundle.w, bundle.g, bundle.W, bundle.ix
    own = ctx is None
    deferred = order == "deferred"
    if own:
        ctx = make_ctx(w, g, W, precision, max(c for _, c in batches), order)
    if warm_at is None:
        st = O.OracleState.zeros(g.num_nodes, w.mem_dim)
        ctx.reset()
    else:
        st = O.OracleState(*S.make_warm_state(w, g, warm_at))
        ctx.state_import(st.mem, st.last_update)
    before = (st.mem.copy(), st.last_update.copy())
    applied = None  # deferred order: the batch whose winners the next step applies
    worst = {}
    for n, (first, count) in enumerate(batches):
        if not quiet or n % 50 == 0:
            print(f"[{w.name} {precision}] step first_eid={first} count={count}", flush=True)
        neg = S.make_negatives(w, g, first, count) if with_neg else None
        if locked:
            ctx.state_import(st.mem, st.last_update)
            st.drop_pending()
            before = (st.mem.copy(), st.last_update.copy())
            applied = None
        ref = O.step(st, g.src, g.dst, g.ts, g.edge_feat, W, first, count, neg, w.num_neighbors,
                     w.num_heads, index=ix, deferred=deferred)
        out = ctx.alloc_outputs(count, with_neg=with_neg, inspect=True)
        ctx.step(first, count, torch.from_numpy(neg).to("cuda:0") if with_neg else None, out)
        torch.cuda.synchronize()
        if expect_launches is not None and n > 0 and not locked:
            assert ctx.launch_info()["kernels_per_step"] == expect_launches
        msg = (first, count) if not deferred else applied
        touched = (np.concatenate([g.src[msg[0]:msg[0] + msg[1]], g.dst[msg[0]:msg[0] + msg[1]]])
                   if msg is not None else np.zeros(0, dtype=np.int64))
        res = compare_step(ctx, out, ref, st, TOL[precision], before=before, touched=touched)
        before = res.pop("state")
        applied = (first, count)
        for k, v in res.items():
            worst[k] = max(worst.get(k, 0.0), v)
    print(f"[{w.name} {precision}] worst gate ratios: {worst}", flush=True)
    if own:
        ctx.close()
    return worst


def window(w, frac, steps, batch=None):
    B = batch or w.batch_size
    first = int(w.num_events * frac) // B * B
    return first, list(S.batches(w.num_events, B, first=first, stop=first + steps * B))


# ------------------------------------------------------------------------------------- C1


@pytest.fixture(scope="module")
def c1():
    return Bundle(S.WORKLOADS["c1_tiny"])


def test_c1_whole_stream_free_running_fp32(c1):
    run(c1, "fp32", list(S.batches(c1.w.num_events, c1.w.batch_size)), locked=False)


def test_c1_step_locked_fp32_ragged_tiles_and_short_tail(c1):
    # batch 136 leaves ragged tiles in both tile kernels; the last batch has 10 events
    run(c1, "fp32", list(S.batches(c1.w.num_events, 136))[:12] + [(9990, 10)], locked=True)


def test_c1_without_negatives(c1):
    run(c1, "fp32", list(S.batches(c1.w.num_events, 200))[:4], locked=False, with_neg=False)


def test_c1_whole_stream_free_running_bf16(c1):
    run(c1, "bf16", list(S.batches(c1.w.num_events, c1.w.batch_size)), locked=False)


def test_c1_single_event_batches(c1):
    run(c1, "fp32", [(e, 1) for e in range(3000, 3006)], locked=False, warm_at=3000)


@pytest.mark.parametrize("precision", ["fp32", "bf16"])
def test_c1_consecutive_batches_prepared_ahead(c1, precision):
    # whole stream incl. the short last batch (10,000 = 73 * 136 + 72), free running: from the second
    # step on a step is two launches, its winners, queries and GRU rows prepared by the step before
    # (the last, shorter batch was anticipated with its real size); and step-locked
    bs = list(S.batches(c1.w.num_events, 136))
    assert bs[-1][1] == 72
    run(c1, precision, bs, locked=False, expect_launches=2)
    run(c1, "fp32", bs[:6], locked=True)


def test_c1_wrong_guesses_of_the_next_batch(c1):
    # batches that do not continue the previous one: revisits, gaps, changing sizes; every step
    # must still equal the oracle's
    import torch
    w, g, W = c1.w, c1.g, c1.W
    ctx = make_ctx(w, g, W, "fp32", 300)
    seq = [(0, 200), (200, 200), (200, 200), (400, 100), (500, 300), (1000, 300), (1300, 300),
           (1600, 7), (1607, 7), (1614, 300), (0, 200), (200, 200)]
    run(c1, "fp32", seq[:5], locked=True, ctx=ctx)
    run(c1, "fp32", seq[5:10], locked=True, ctx=ctx)
    run(c1, "fp32", seq[10:], locked=False, ctx=ctx)   # reset in between
    run(c1, "fp32", [(400, 200), (600, 200)], locked=True, ctx=ctx)
    ctx.close()


@pytest.mark.parametrize("precision", ["fp32", "bf16"])
def test_c1_deferred_order_whole_stream(c1, precision):
    # the step applies the previous batch's winners, embeds, keeps its own; incl. the short last batch
    bs = list(S.batches(c1.w.num_events, 136))
    run(c1, precision, bs, locked=False, order="deferred")
    run(c1, precision, bs[:8], locked=False, order="deferred", with_neg=False)


def test_c1_deferred_order_gaps_sizes_and_imports(c1):
    # batches of changing size with gaps; a state import in between drops what is kept
    ctx = make_ctx(c1.w, c1.g, c1.W, "fp32", 300, "deferred")
    run(c1, "fp32", [(0, 200), (200, 200), (500, 300), (1000, 7), (1007, 7), (1014, 300)], locked=False,
        ctx=ctx, order="deferred")
    run(c1, "fp32", [(3000, 100), (3100, 100), (3200, 100)], locked=False, warm_at=3000, ctx=ctx,
        order="deferred")
    run(c1, "fp32", [(4000, 100), (4100, 100)], locked=True, warm_at=4000, ctx=ctx, order="deferred")
    ctx.close()


# ------------------------------------------------------------------------------------- C2


@pytest.fixture(scope="module")
def c2():
    return Bundle(S.WORKLOADS["c2_bipartite_medium"])


def test_c2_from_reset_free_running_fp32(c2):
    run(c2, "fp32", list(S.batches(c2.w.num_events, 200))[:12], locked=False)


def test_c2_windows_and_last_short_batch_fp32(c2):
    w = c2.w
    for frac in (0.5, 0.9):
        first, bs = window(w, frac, 3)
        run(c2, "fp32", bs, locked=False, warm_at=first)
    last = (w.num_events // 200) * 200            # 157,474 = 787 * 200 + 74
    assert w.num_events - last == 74
    run(c2, "fp32", [(last - 200, 200), (last, 74)], locked=True, warm_at=last - 200)


@pytest.mark.timeout(900)
def test_c2_whole_stream_free_running_fp32(c2):
    # all 788 batches from reset (the last one has 74 events), both sides free running: every step's
    # neighbour tables, winners, embeddings, scores and state; from the second step on two launches
    run(c2, "fp32", list(S.batches(c2.w.num_events, 200)), locked=False, expect_launches=2, quiet=True)


def test_c2_window_bf16(c2):
    first, bs = window(c2.w, 0.5, 3)
    run(c2, "bf16", bs, locked=False, warm_at=first, expect_launches=2)


# ------------------------------------------------------------------------------------- C3


@pytest.fixture(scope="module")
def c3():
    return Bundle(S.WORKLOADS["c3_bipartite_dense"])


@pytest.mark.parametrize("precision", ["fp32", "bf16"])
@pytest.mark.parametrize("batch", [200, 2000])
def test_c3_windows(c3, precision, batch):
    steps = 3 if batch == 200 else 2
    for frac in (0.1, 0.5, 0.9):
        first, bs = window(c3.w, frac, steps, batch)
        run(c3, precision, bs, locked=False, warm_at=first)


def test_c3_batch_above_the_fused_selection_limit(c3):
    # more than 4096 events per batch: the winner selection runs as a launch of its own
    first, bs = window(c3.w, 0.5, 1, 5000)
    run(c3, "fp32", bs, locked=False, warm_at=first)
    # ... and is never done ahead; 4096 -> 5000 -> 3000 crosses the limit in both directions
    first, bs = window(c3.w, 0.5, 1, 4096)
    seq = bs + [(first + 4096, 5000), (first + 9096, 3000), (first + 12096, 3000)]
    run(c3, "fp32", seq, locked=False, warm_at=first)
    run(c3, "fp32", seq, locked=False, warm_at=first, order="deferred")
    # three large batches in a row (their keys stay in the per-node arrays from one to the next),
    # then a state import and a restart from an earlier event
    ctx = make_ctx(c3.w, c3.g, c3.W, "fp32", 5000, "deferred")
    big = [(first + i * 5000, 5000) for i in range(3)]
    run(c3, "fp32", big, locked=False, warm_at=first, ctx=ctx, order="deferred")
    run(c3, "fp32", [(first - 3000, 3000), (first, 5000)], locked=False, warm_at=first - 3000, ctx=ctx,
        order="deferred")
    ctx.close()
    ctx = make_ctx(c3.w, c3.g, c3.W, "fp32", 5000)
    run(c3, "fp32", big, locked=False, warm_at=first, ctx=ctx)
    run(c3, "fp32", [(first - 3000, 3000), (first, 5000)], locked=False, warm_at=first - 3000, ctx=ctx)
    ctx.close()


# ------------------------------------------------------------------------------------- C4


@pytest.fixture(scope="module")
def c4():
    return Bundle(S.WORKLOADS["c4_million_node"])


@pytest.mark.timeout(600)
@pytest.mark.parametrize("precision", ["bf16", "fp32"])
def test_c4_windows(c4, precision):
    for frac in (0.1, 0.9):
        first, bs = window(c4.w, frac, 2)
        run(c4, precision, bs, locked=False, warm_at=first)
