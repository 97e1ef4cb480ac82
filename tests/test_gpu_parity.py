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


def _ctx(w, g, W, precision, max_batch=None):
    import torch
    from paper_2308_14129_amd import tig
    assert torch.cuda.is_available()
    cfg = tig.make_config(w.mem_dim, w.time_dim, w.feat_dim, w.emb_dim, w.num_neighbors, w.num_heads,
                          max_batch or w.batch_size, precision)
    return tig.TigContext(cfg, g.num_nodes, g.src, g.dst, g.ts, g.edge_feat, W, device="cuda:0")


def _run(w, precision, batches, locked, state0=None, with_neg=True, g=None, W=None, ix=None):
    """Runs the batches on both sides.  locked=True loads the oracle's state into the GPU before
    every step (step-locked parity); otherwise both sides run freely from the same start."""
    import torch
    g = g if g is not None else S.make_graph(w)
    W = W if W is not None else S.make_weights(w)
    ix = ix if ix is not None else O.NeighbourIndex(g.num_nodes, g.src, g.dst, g.ts)
    ctx = _ctx(w, g, W, precision, max(c for _, c in batches))
    st = O.OracleState.zeros(g.num_nodes, w.mem_dim) if state0 is None else state0
    if state0 is not None:
        ctx.state_import(st.mem, st.last_update)
    worst = {}
    for first, count in batches:
        print(f"[{w.name} {precision}] step first_eid={first} count={count}", flush=True)
        neg = S.make_negatives(w, g, first, count) if with_neg else None
        if locked:
            ctx.state_import(st.mem, st.last_update)
        ref = O.step(st, g.src, g.dst, g.ts, g.edge_feat, W, first, count, neg, w.num_neighbors,
                     w.num_heads, index=ix)
        out = ctx.alloc_outputs(count, with_neg=with_neg, inspect=True)
        ctx.step(first, count, torch.from_numpy(neg).to("cuda:0") if with_neg else None, out)
        torch.cuda.synchronize()
        res = compare_step(ctx, out, ref, st, TOL[precision])
        for k, v in res.items():
            worst[k] = max(worst.get(k, 0.0), v)
    print(f"[{w.name} {precision}] worst gate ratios: {worst}", flush=True)
    ctx.close()
    return worst


def test_c1_tiny_whole_stream_free_running_fp32():
    w = S.WORKLOADS["c1_tiny"]
    _run(w, "fp32", list(S.batches(w.num_events, w.batch_size)), locked=False)


def test_c1_tiny_step_locked_fp32_and_ragged_tail():
    w = S.WORKLOADS["c1_tiny"]
    # batch 136 leaves ragged tiles in both tile kernels and a short last batch
    _run(w, "fp32", list(S.batches(w.num_events, 136))[:12] + [(9990, 10)], locked=True)


def test_c1_tiny_without_negatives():
    w = S.WORKLOADS["c1_tiny"]
    _run(w, "fp32", list(S.batches(w.num_events, 200))[:4], locked=False, with_neg=False)
