"""Comparison helpers for the GPU-vs-oracle parity tests."""
from __future__ import annotations

import numpy as np


def gate(got: np.ndarray, ref: np.ndarray, tol: float, name: str) -> float:
    """Tolerance gate per tensor: |got - ref| <= tol * (|ref| + mean|ref|), element-wise.
    Returns the largest ratio |got - ref| / (|ref| + mean|ref|)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, f"{name}: shape {got.shape} vs {ref.shape}"
    assert np.all(np.isfinite(got)), f"{name}: non-finite values in the GPU result"
    if ref.size == 0:
        return 0.0
    s = float(np.mean(np.abs(ref)))
    denom = np.abs(ref) + s
    denom[denom == 0.0] = 1.0
    ratio = np.abs(got - ref) / denom
    worst = float(ratio.max())
    assert worst <= tol, (f"{name}: max |got-ref|/(|ref|+mean|ref|) = {worst:.3e} > {tol:g} "
                          f"(max abs err {np.abs(got - ref).max():.3e}, mean|ref| {s:.3e})")
    return worst


def compare_step(ctx, out, ref, oracle_state, tol, check_state=True):
    """Neighbour tables and winners bit-exact; embeddings, scores and state within `tol`.
    Without the per-entry winner flags the winners are still pinned through last_update, which
    must equal the oracle's bit for bit over all nodes."""
    np.testing.assert_array_equal(out.nbr_cnt.cpu().numpy(), ref["nbr_cnt"], err_msg="nbr_cnt")
    np.testing.assert_array_equal(out.nbr_node.cpu().numpy(), ref["nbr_node"], err_msg="nbr_node")
    np.testing.assert_array_equal(out.nbr_eid.cpu().numpy(), ref["nbr_eid"], err_msg="nbr_eid")
    np.testing.assert_array_equal(out.nbr_ts.cpu().numpy(), ref["nbr_ts"], err_msg="nbr_ts")
    if out.is_winner is not None:
        np.testing.assert_array_equal(out.is_winner.cpu().numpy(), ref["is_winner"], err_msg="is_winner")
    res = {"emb": gate(out.emb.cpu().numpy(), ref["emb"], tol, "emb"),
           "score_pos": gate(out.score_pos.cpu().numpy(), ref["score_pos"], tol, "score_pos")}
    if ref["score_neg"] is not None:
        res["score_neg"] = gate(out.score_neg.cpu().numpy(), ref["score_neg"], tol, "score_neg")
    if check_state:
        mem, lu = ctx.state_export()
        np.testing.assert_array_equal(lu, oracle_state.last_update, err_msg="last_update")
        res["mem"] = gate(mem, oracle_state.mem, tol, "mem")
        # rows the oracle left untouched must be bit-identical on the GPU as well
    return res
