"""tig_step_static (the step with its intermediates in the library's static device array, for
callers that cannot allocate) against tig_step on a twin context: same kernels on the same
inputs, so every output and the state must agree bit for bit.  Two calls in a row, the second
with a smaller batch; then both again after the array has been used by another configuration."""
import ctypes

import numpy as np
import pytest

import tig_synth as S
from tests.test_gpu_parity import Bundle, make_ctx

pytestmark = pytest.mark.gpu

NAMES = ("emb", "score_pos", "score_neg", "nbr_node", "nbr_eid", "nbr_ts", "nbr_cnt", "is_winner")


def _twin_steps(bundle, precision, seq, warm_at, static_calls=None):
    import torch
    w, g, W = bundle.w, bundle.g, bundle.W
    ref_ctx = make_ctx(w, g, W, precision, max(c for _, c in seq))
    new_ctx = make_ctx(w, g, W, precision, max(c for _, c in seq))
    warm = S.make_warm_state(w, g, warm_at)
    ref_ctx.state_import(*warm)
    new_ctx.state_import(*warm)
    for first, count in seq:
        print(f"[static] {w.name} {precision} first_eid={first} count={count}", flush=True)
        neg = torch.from_numpy(S.make_negatives(w, g, first, count)).to("cuda:0")
        a = ref_ctx.alloc_outputs(count, inspect=True)
        b = new_ctx.alloc_outputs(count, inspect=True)
        ref_ctx.step(first, count, neg, a)
        new_ctx.step(first, count, neg, b, static=static_calls is None or (first, count) in static_calls)
        torch.cuda.synchronize()
        for n in NAMES:
            assert torch.equal(getattr(a, n), getattr(b, n)), n
        ma, la = ref_ctx.state_export()
        mb, lb = new_ctx.state_export()
        assert np.array_equal(ma, mb) and np.array_equal(la, lb)
    ref_ctx.close()
    new_ctx.close()


def test_static_scratch_step_equals_tig_step():
    c1 = Bundle(S.WORKLOADS["c1_tiny"])
    # two calls in a row, the second smaller; then a gap and a larger one again
    _twin_steps(c1, "fp32", [(3000, 200), (3200, 72), (3300, 1), (3400, 200)], warm_at=3000)
    # another configuration leaves other contents in the array; then the first one again
    odd = Bundle(S.Workload(name="odd", index=7, n_src=300, n_dst=0, num_events=3000, alpha_src=1.2,
                            alpha_dst=1.2, span=500.0, integer_seconds=True, feat_dim=40, mem_dim=100,
                            time_dim=60, emb_dim=48, num_neighbors=16, num_heads=4, batch_size=100,
                            precision="bf16"))
    _twin_steps(odd, "bf16", [(1000, 100), (1100, 37)], warm_at=1000)
    _twin_steps(c1, "bf16", [(5000, 136), (5136, 50)], warm_at=5000)


def test_static_and_ordinary_steps_mixed_on_one_context():
    # consecutive batches, so every ordinary step prepares the next batch (winners, queries, GRU
    # rows); a static call in between uses none of it and changes the memory under it
    c1 = Bundle(S.WORKLOADS["c1_tiny"])
    seq = [(4000 + 136 * i, 136) for i in range(7)]
    _twin_steps(c1, "fp32", seq, warm_at=4000, static_calls={seq[2], seq[3], seq[5]})


def test_static_scratch_step_rejects_what_it_cannot_hold():
    from paper_2308_14129_amd import tig
    c1 = Bundle(S.WORKLOADS["c1_tiny"])
    w, g, W = c1.w, c1.g, c1.W
    import torch
    neg = torch.from_numpy(S.make_negatives(w, g, 0, 200)).to("cuda:0")
    # intermediates beyond the static array: 65536 events x 64 neighbours
    cfg = tig.make_config(w.mem_dim, w.time_dim, w.feat_dim, w.emb_dim, 64, w.num_heads, 65536, "fp32")
    big = tig.TigContext(cfg, g.num_nodes, g.src, g.dst, g.ts, g.edge_feat, W)
    out = big.alloc_outputs(200)
    with pytest.raises(tig.TigError) as ei:
        big.step(0, 200, neg, out, static=True)
    assert ei.value.status == tig.TIG_ENOSPACE
    assert b"TIG_STATIC_SCRATCH_BYTES" in big.lib.tig_last_error(big.handle)
    mem, lu = big.state_export()
    assert not mem.any() and not lu.any()                     # nothing ran
    big.step(0, 200, neg, out)                                # the ordinary step still works
    torch.cuda.synchronize()
    big.close()
    # deferred contexts keep their pending winners in the context's own scratch: refused
    d = make_ctx(w, g, W, "fp32", 200, "deferred")
    with pytest.raises(tig.TigError) as ei:
        d.step(0, 200, neg, d.alloc_outputs(200), static=True)
    assert ei.value.status == tig.TIG_EINVAL
    d.close()
