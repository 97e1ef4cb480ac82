"""Where the time goes inside the two tile kernels of a step: per-workgroup timestamps at the phase
boundaries, from the instrumented build of the library.

    python -m paper_2308_14129_amd.build --phase-clocks          # builds libtig_clocks.so (no GPU needed)
    python -m paper_2308_14129_amd.phase_clocks [workload] [fp32|bf16] [batch]

Runs 12 consecutive steps of the workload's mid-stream window on the instrumented library and prints,
for the last step: the embedding launch's phases (A rows, B query fold, C attention, D merge layer 1,
E merge layer 2 + decoder halves) over its row tiles, its side workgroups, and the closing launch's GRU
workgroups, event blocks and finishing blocks.  Times are in microseconds of the 100 MHz device clock."""
from __future__ import annotations

import ctypes
import os
import sys

import numpy as np


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    sys.path.insert(0, os.path.dirname(here))
    import torch
    import tig_synth as S
    from paper_2308_14129_amd import tig
    assert tig._lib is None, "the library is already loaded"
    tig.LIB_PATH = os.path.join(here, "libtig_clocks.so")   # the instrumented build

    name = sys.argv[1] if len(sys.argv) > 1 else "c5_gpu_partition"
    prec = sys.argv[2] if len(sys.argv) > 2 else "bf16"
    w = S.WORKLOADS[name]
    B = int(sys.argv[3]) if len(sys.argv) > 3 else w.batch_size
    g, W = S.make_graph(w), S.make_weights(w)
    cfg = tig.make_config(w.mem_dim, w.time_dim, w.feat_dim, w.emb_dim, w.num_neighbors, w.num_heads, B, prec)
    ctx = tig.TigContext(cfg, g.num_nodes, g.src, g.dst, g.ts, g.edge_feat, W)
    first = (w.num_events // 2) // B * B
    ctx.state_import(*S.make_warm_state(w, g, first))
    out = ctx.alloc_outputs(B)
    for i in range(12):
        f = first + i * B
        ctx.step(f, B, torch.from_numpy(S.make_negatives(w, g, f, B)).cuda(), out)
    torch.cuda.synchronize()

    def clocks(symbol, blocks):
        buf = np.zeros(blocks * 8, dtype=np.uint64)
        assert getattr(ctx.lib, symbol)(ctypes.c_void_p(buf.ctypes.data), blocks * 8) == 0
        c = buf.reshape(blocks, 8).astype(np.int64)
        c[c[:, 0] <= c.max() - 20000] = 0   # marks of earlier launches
        return c

    us = lambda ticks: ticks * 0.01
    c = clocks("tig_debug_phase_clocks", 1024)
    tile = (c[:, 5] > 0) & (c[:, 0] > 0) & (c[:, 7] == 0)
    side = (c[:, 7] > 0) & (c[:, 0] > 0) & (c[:, 5] == 0)
    ct = c[tile]
    t0 = ct[:, 0].min()
    d = us(np.diff(ct[:, :6], axis=1))
    print(f"{name} {prec} batch {B}")
    print(f"embedding launch: {int(tile.sum())} row tiles in use, {int(side.sum())} side workgroups")
    print("  phases A B C D E, mean us:", np.round(d.mean(axis=0), 2), " slowest tile:", np.round(d.max(axis=0), 2))
    print(f"  tiles start {us(ct[:, 0] - t0).mean():.2f} (mean) after the first, the last ends at {us(ct[:, 5] - t0).max():.2f}")
    cs = c[side]
    if len(cs):
        print(f"  side workgroups (selection, query preparation): mean {us(cs[:, 7] - cs[:, 0]).mean():.2f}, "
              f"last ends at {us(cs[:, 7] - t0).max():.2f}")
    nb = 2048
    c = clocks("tig_debug_phase_clocks_gru", nb)
    t0 = c[:, 0][c[:, 0] > 0].min()
    gru = (c[:, 0] > 0) & (c[:, 1] > c[:, 0]) & (c[:, 2] > c[:, 1]) & (c[:, 3] > c[:, 2]) & (c[:, 4] >= c[:, 3])
    cg = c[gru]
    d = us(np.diff(cg[:, :5], axis=1))
    print(f"closing launch: {int(gru.sum())} GRU workgroups with work")
    print("  descriptors, gather, gates, epilogue, mean us:", np.round(d.mean(axis=0), 2), f" last ends at {us(cg[:, 4] - t0).max():.2f}")
    n_gru, n_ev = 256, (B + 7) // 8
    idx = np.arange(nb)
    for label, lo, hi in (("event blocks", n_gru, n_gru + n_ev), ("finishing blocks", n_gru + n_ev, n_gru + n_ev + 144)):
        sel = (idx >= lo) & (idx < hi) & (c[:, 0] > 0) & (c[:, 1] >= c[:, 0])
        cf = c[sel]
        if len(cf):
            print(f"  {label}: {int(sel.sum())}, mean {us(cf[:, 1] - cf[:, 0]).mean():.2f} us each, last ends at {us(cf[:, 1] - t0).max():.2f}")
    ctx.close()


if __name__ == "__main__":
    main()
