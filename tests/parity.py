"""Comparison helpers for the GPU-vs-oracle parity tests."""
from __future__ import annotations

import os

import numpy as np

REPORT = os.environ.get("TIG_PARITY_REPORT", "") not in ("", "0")   # also print max abs and pure-relative errors


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
    if REPORT:
        big = np.abs(ref) > 1e-3 * max(s, 1e-30)   # pure relative error where the reference is not near zero
        rel = float((np.abs(got - ref)[big] / np.abs(ref)[big]).max()) if big.any() else 0.0
        print(f"[gate] {name}: ratio {worst:.2e} (tol {tol:g}), max abs {np.abs(got - ref).max():.2e}, "
              f"max relative (|ref| > 1e-3 mean|ref|) {rel:.2e}", flush=True)
    assert worst <= tol, (f"{name}: max |got-ref|/(|ref|+mean|ref|) = {worst:.3e} > {tol:g} "
                          f"(max abs err {np.abs(got - ref).max():.3e}, mean|ref| {s:.3e})")
    return worst


def compare_step(ctx, out, ref, oracle_state, tol, check_state=True, before=None, touched=None):
    """Neighbour tables and winners bit-exact; embeddings, scores and state within `tol`.
    before = (mem, last_update) of the GPU side when the step started and touched = the node ids
    whose messages the step applied: every other row must come out of the step bit-identical.
    Returns the gate ratios and, under "state", the exported (mem, last_update)."""
    np.testing.assert_array_equal(out.nbr_cnt.cpu().numpy(), ref["nbr_cnt"], err_msg="nbr_cnt")
    np.testing.assert_array_equal(out.nbr_node.cpu().numpy(), ref["nbr_node"], err_msg="nbr_node")
    np.testing.assert_array_equal(out.nbr_eid.cpu().numpy(), ref["nbr_eid"], err_msg="nbr_eid")
    np.testing.assert_array_equal(out.nbr_ts.cpu().numpy(), ref["nbr_ts"], err_msg="nbr_ts")
    np.testing.assert_array_equal(out.is_winner.cpu().numpy(), ref["is_winner"], err_msg="is_winner")
    res = {"emb": gate(out.emb.cpu().numpy(), ref["emb"], tol, "emb"),
           "score_pos": gate(out.score_pos.cpu().numpy(), ref["score_pos"], tol, "score_pos")}
    if ref["score_neg"] is not None:
        res["score_neg"] = gate(out.score_neg.cpu().numpy(), ref["score_neg"], tol, "score_neg")
    if check_state:
        mem, lu = ctx.state_export()
        np.testing.assert_array_equal(lu, oracle_state.last_update, err_msg="last_update")
        res["mem"] = gate(mem, oracle_state.mem, tol, "mem")
        if before is not None:
            keep = np.ones(mem.shape[0], dtype=bool)
            keep[np.asarray(touched, dtype=np.int64)] = False
            assert np.array_equal(mem[keep], before[0][keep]), "a memory row outside the applied batch changed"
            assert np.array_equal(lu[keep], before[1][keep]), "last_update outside the applied batch changed"
        res["state"] = (mem, lu)
    return res
