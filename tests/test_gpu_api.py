"""Boundary behaviour on the GPU: error codes, reset / export / import, determinism, invariants,
degenerate graphs and odd shapes."""
import ctypes

import numpy as np
import pytest

import tig_synth as S
from oracle import tig_oracle as O
from tests.parity import compare_step
from tests.test_gpu_parity import Bundle, make_ctx, run

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def c1():
    return Bundle(S.WORKLOADS["c1_tiny"])


def _init_status(w, g, W, **over):
    from paper_2308_14129_amd import tig
    src, dst, ts = over.get("src", g.src), over.get("dst", g.dst), over.get("ts", g.ts)
    cfg = tig.make_config(w.mem_dim, w.time_dim, w.feat_dim, w.emb_dim, w.num_neighbors, w.num_heads, 200)
    try:
        ctx = tig.TigContext(cfg, g.num_nodes, src, dst, ts, g.edge_feat, W)
    except tig.TigError as e:
        return e.status
    ctx.close()
    return 0


def test_init_rejects_bad_graphs(c1):
    from paper_2308_14129_amd import tig
    w, g, W = c1.w, c1.g, c1.W
    ts = g.ts.copy()
    ts[5000] = ts[4999] - 1.0
    assert _init_status(w, g, W, ts=ts) == tig.TIG_EUNSORTED
    src = g.src.copy()
    src[77] = g.dst[77]
    assert _init_status(w, g, W, src=src) == tig.TIG_ESELFLOOP
    dst = g.dst.copy()
    dst[9999] = g.num_nodes
    assert _init_status(w, g, W, dst=dst) == tig.TIG_ERANGE
    src = g.src.copy()
    src[0] = -1
    assert _init_status(w, g, W, src=src) == tig.TIG_ERANGE
    assert _init_status(w, g, W) == 0


def test_init_rejects_small_workspace_and_null(c1):
    import torch
    from paper_2308_14129_amd import tig
    w, g, W = c1.w, c1.g, c1.W
    lib = tig.load_library()
    cfg = tig.make_config(w.mem_dim, w.time_dim, w.feat_dim, w.emb_dim, w.num_neighbors, w.num_heads, 200)
    p, s = tig.workspace_bytes(cfg, g.num_nodes, g.num_events)
    pers = torch.empty(p, dtype=torch.uint8, device="cuda:0")
    scr = torch.empty(s, dtype=torch.uint8, device="cuda:0")
    gg = tig.tig_graph(ctypes.sizeof(tig.tig_graph), 0, g.num_nodes, g.num_events, g.src.ctypes.data,
                       g.dst.ctypes.data, g.ts.ctypes.data, g.edge_feat.ctypes.data)
    ww = tig.tig_weights(ctypes.sizeof(tig.tig_weights), 0, *[W[n].ctypes.data for n in tig.WEIGHT_NAMES])
    h = ctypes.c_void_p(None)
    args = lambda pb, sb: (ctypes.byref(cfg), ctypes.byref(gg), ctypes.byref(ww), pers.data_ptr(), pb,
                           scr.data_ptr(), sb, None, ctypes.byref(h))
    assert lib.tig_init(*args(p - 1, s)) == tig.TIG_ENOSPACE and not h.value
    assert lib.tig_init(*args(p, s - 1)) == tig.TIG_ENOSPACE and not h.value
    ww.W_K = None
    assert lib.tig_init(*args(p, s)) == tig.TIG_EINVAL and not h.value


def test_step_argument_errors_leave_state_unchanged(c1):
    import torch
    from paper_2308_14129_amd import tig
    w, g, W = c1.w, c1.g, c1.W
    ctx = make_ctx(w, g, W, "fp32")
    mem0, lu0 = S.make_warm_state(w, g, 5000)
    ctx.state_import(mem0, lu0)
    out = ctx.alloc_outputs(200, with_neg=True)
    neg = torch.from_numpy(S.make_negatives(w, g, 5000, 200)).to("cuda:0")
    sz_b, sz_o = ctypes.sizeof(tig.tig_batch), ctypes.sizeof(tig.tig_out)
    good_o = tig.tig_out(sz_o, 0, out.emb.data_ptr(), out.score_pos.data_ptr(), out.score_neg.data_ptr(),
                         None, None, None, None, None)
    cases = [
        (tig.tig_batch(sz_b, 201, 5000, neg.data_ptr()), good_o, tig.TIG_EINVAL),      # count > max_batch
        (tig.tig_batch(sz_b, 0, 5000, neg.data_ptr()), good_o, tig.TIG_EINVAL),
        (tig.tig_batch(sz_b, 200, 9900, neg.data_ptr()), good_o, tig.TIG_ERANGE),      # leaves the graph
        (tig.tig_batch(sz_b, 200, -1, neg.data_ptr()), good_o, tig.TIG_ERANGE),
        (tig.tig_batch(sz_b - 4, 200, 5000, neg.data_ptr()), good_o, tig.TIG_EINVAL),  # struct_size
        (tig.tig_batch(sz_b, 200, 5000, neg.data_ptr()),
         tig.tig_out(sz_o, 0, None, out.score_pos.data_ptr(), out.score_neg.data_ptr(), None, None, None, None, None),
         tig.TIG_EINVAL),
        (tig.tig_batch(sz_b, 200, 5000, neg.data_ptr()),
         tig.tig_out(sz_o, 0, out.emb.data_ptr(), out.score_pos.data_ptr(), None, None, None, None, None, None),
         tig.TIG_EINVAL),                                                             # negatives without score_neg
    ]
    for b, o, want in cases:
        assert ctx.step_raw(b, o) == want
        assert ctx.lib.tig_last_error(ctx.handle) != b""
    mem1, lu1 = ctx.state_export()
    assert np.array_equal(mem0, mem1) and np.array_equal(lu0, lu1)
    # chronological order: after a step over [5000, 5200) a batch may start at 5200 or later, not
    # before, until a reset or an import rewinds the cursor
    good_b = tig.tig_batch(sz_b, 200, 5000, neg.data_ptr())
    assert ctx.step_raw(good_b, good_o) == tig.TIG_OK
    torch.cuda.synchronize()
    mem2, lu2 = ctx.state_export()
    for first in (5000, 5199, 0):
        assert ctx.step_raw(tig.tig_batch(sz_b, 100, first, neg.data_ptr()), good_o) == tig.TIG_EORDER
    mem3, lu3 = ctx.state_export()
    assert np.array_equal(mem2, mem3) and np.array_equal(lu2, lu3)
    assert ctx.step_raw(tig.tig_batch(sz_b, 100, 5300, neg.data_ptr()), good_o) == tig.TIG_OK   # gaps are fine
    ctx.state_import(mem0, lu0)
    assert ctx.step_raw(good_b, good_o) == tig.TIG_OK
    ctx.reset()
    assert ctx.step_raw(tig.tig_batch(sz_b, 100, 0, neg.data_ptr()), good_o) == tig.TIG_OK
    torch.cuda.synchronize()
    ctx.close()


def test_reset_export_import_roundtrip_and_determinism(c1):
    import torch
    w, g, W = c1.w, c1.g, c1.W
    ctx = make_ctx(w, g, W, "fp32")
    mem, lu = ctx.state_export()
    assert not mem.any() and not lu.any()                       # state after tig_init = after a reset
    batches = list(S.batches(g.num_events, 200))[10:14]

    def play():
        outs = []
        for first, count in batches:
            neg = torch.from_numpy(S.make_negatives(w, g, first, count)).to("cuda:0")
            o = ctx.alloc_outputs(count, inspect=True)
            ctx.step(first, count, neg, o)
            outs.append(o)
        torch.cuda.synchronize()
        return outs, ctx.state_export()

    warm = S.make_warm_state(w, g, batches[0][0])
    ctx.state_import(*warm)
    m, l = ctx.state_export()
    assert np.array_equal(m, warm[0]) and np.array_equal(l, warm[1])      # import -> export
    o1, s1 = play()
    ctx.state_import(*warm)
    o2, s2 = play()
    # identical inputs give bit-identical outputs and state (the atomicMax keys make the winner
    # choice independent of scheduling)
    assert np.array_equal(s1[0], s2[0]) and np.array_equal(s1[1], s2[1])
    for a, b in zip(o1, o2):
        for name in ("emb", "score_pos", "score_neg", "nbr_node", "nbr_eid", "nbr_ts", "nbr_cnt", "is_winner"):
            assert torch.equal(getattr(a, name), getattr(b, name)), name
    # export -> import -> step == step (device-pointer import path)
    ctx.state_import(*warm)
    play_first = batches[0]
    neg = torch.from_numpy(S.make_negatives(w, g, *play_first)).to("cuda:0")
    o = ctx.alloc_outputs(play_first[1])
    dm = torch.from_numpy(warm[0]).to("cuda:0")
    dl = torch.from_numpy(warm[1]).to("cuda:0")
    ctx.state_import(dm, dl)
    ctx.step(play_first[0], play_first[1], neg, o)
    torch.cuda.synchronize()
    assert torch.equal(o.emb, o1[0].emb)
    ctx.reset()
    mem, lu = ctx.state_export()
    assert not mem.any() and not lu.any()
    ctx.close()


def test_launches_per_step(c1):
    """A step whose batch continues the previous one runs two kernels (its winners and queries
    were prepared inside the previous embedding launch, its GRU rows by the previous closing
    launch); any other step prepares them in two launches of its own.  Asking for the inspection
    outputs does not change what is launched."""
    import torch
    w, g, W = c1.w, c1.g, c1.W
    ctx = make_ctx(w, g, W, "fp32")
    assert ctx.launch_info()["kernels_per_step"] == 0
    out = ctx.alloc_outputs(200)
    flagged = ctx.alloc_outputs(200, inspect=True)
    seen = []
    for first, o in ((0, out), (200, out), (400, out), (800, out), (1000, flagged), (1200, out)):
        neg = torch.from_numpy(S.make_negatives(w, g, first, 200)).to("cuda:0")
        ctx.step(first, 200, neg, o)
        seen.append(ctx.launch_info()["kernels_per_step"])
    torch.cuda.synchronize()
    # first step; two that continue; a gap; one that asks for the winner flags; one that continues
    assert seen == [4, 2, 2, 4, 2, 2]
    ctx.close()


def test_untouched_rows_are_bit_identical(c1):
    import torch
    w, g, W = c1.w, c1.g, c1.W
    ctx = make_ctx(w, g, W, "fp32")
    mem0, lu0 = S.make_warm_state(w, g, 8000)
    ctx.state_import(mem0, lu0)
    out = ctx.alloc_outputs(200)
    neg = torch.from_numpy(S.make_negatives(w, g, 8000, 200)).to("cuda:0")
    ctx.step(8000, 200, neg, out)
    torch.cuda.synchronize()
    mem1, lu1 = ctx.state_export()
    touched = np.zeros(g.num_nodes, dtype=bool)
    touched[g.src[8000:8200]] = True
    touched[g.dst[8000:8200]] = True
    assert np.array_equal(mem1[~touched], mem0[~touched]) and np.array_equal(lu1[~touched], lu0[~touched])
    assert np.all(lu1[touched] >= g.ts[8000])
    ctx.close()


def _custom(name, **kw):
    base = dict(name=name, index=7, n_src=300, n_dst=0, num_events=3000, alpha_src=1.2, alpha_dst=1.2,
                span=500.0, integer_seconds=True, feat_dim=16, mem_dim=32, time_dim=16, emb_dim=32,
                num_neighbors=10, num_heads=2, batch_size=100, precision="fp32")
    base.update(kw)
    return Bundle(S.Workload(**base))


@pytest.mark.parametrize("shape", [
    dict(mem_dim=7, time_dim=5, feat_dim=3, emb_dim=9, num_heads=1, num_neighbors=3),
    dict(mem_dim=33, time_dim=31, feat_dim=1, emb_dim=17, num_heads=4, num_neighbors=64),
    dict(mem_dim=200, time_dim=56, feat_dim=256, emb_dim=130, num_heads=2, num_neighbors=5, batch_size=70),
    # rows with a full set of neighbours take the across-lanes softmax: four heads (two score
    # registers), and sixteen slots in one chunk (eight slot pairs per register row)
    dict(mem_dim=100, time_dim=60, feat_dim=40, emb_dim=48, num_heads=4, num_neighbors=10, alpha_src=2.0),
    dict(mem_dim=32, time_dim=16, feat_dim=16, emb_dim=32, num_heads=2, num_neighbors=16, alpha_src=2.0),
])
@pytest.mark.parametrize("precision", ["fp32", "bf16"])
def test_odd_shapes(shape, precision):
    b = _custom("odd", **shape)
    run(b, precision, list(S.batches(b.w.num_events, b.w.batch_size))[10:14], locked=False, warm_at=10 * b.w.batch_size)


def test_hub_in_every_event_and_heavy_ties():
    """Node 0 takes part in every event (one winner among 2B entries for it) and timestamps are
    whole seconds with ~6 events per second, so strict-earlier and tie order are exercised."""
    b = _custom("hub", alpha_src=8.0, span=500.0)
    deg0 = np.bincount(np.concatenate([b.g.src, b.g.dst]), minlength=b.w.n_src)[0]
    assert deg0 > 0.9 * b.w.num_events
    run(b, "fp32", list(S.batches(b.w.num_events, 100))[5:9], locked=False, warm_at=500)


def test_all_equal_timestamps_give_empty_neighbourhoods():
    import torch
    b = _custom("flat", span=0.5)                   # floor(t) = 0 for every event
    assert not b.g.ts.any()
    ctx = make_ctx(b.w, b.g, b.W, "fp32")
    out = ctx.alloc_outputs(100, inspect=True)
    neg = torch.from_numpy(S.make_negatives(b.w, b.g, 1000, 100)).to("cuda:0")
    ctx.step(1000, 100, neg, out)
    torch.cuda.synchronize()
    assert int(out.nbr_cnt.abs().sum()) == 0 and int((out.nbr_node != -1).sum()) == 0
    ctx.close()
    run(b, "fp32", [(1000, 100)], locked=False, warm_at=1000)
