#!/usr/bin/env python3
"""Benchmark of the TIG batch step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--precision fp32|bf16]

A "step" is one tig_step call: the whole hot path (winner selection, neighbour lookup, message +
GRU, memory overwrite, attention embedding + decoder) over one chronological batch of the
synthetic workload.  The graph, the warm state and every batch's negatives are resident in HBM
before the timed region starts.  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X HBM3E, published
BF16_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA, published
FP32_MFMA_PEAK_TFLOPS = 157.3

PROFILES = os.path.join(ROOT, "profiles")


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def profile_figures(kind, workload, precision, batch):
    """key: value lines of profiles/<kind>_<workload>_<precision>.md (written by
    paper_2308_14129_amd.profiling from the rocprofv3 runs described there); {} if there is no such
    file, it is for another batch size, or the kernel sources have changed since it was measured."""
    from paper_2308_14129_amd.profiling import kernel_source_id
    path = os.path.join(PROFILES, f"{kind}_{workload}_{precision}.md")
    if not os.path.exists(path):
        return {}
    vals = {}
    for line in open(path):
        line = line.strip()
        if line.startswith("- `") and "`:" in line:
            k, v = line[3:].split("`:", 1)
            vals[k.strip()] = v.strip()
    if vals.get("kernel_source_id") != kernel_source_id() or vals.get("batch") != str(batch):
        return {}
    return vals


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def oracle_baseline(g, w, weights, batches, negs_np, mem0, lu0, order, n_steps, workers):
    """The oracle as it stands on the host cores: (i) one thread, n_steps consecutive steps of the
    timed window; (ii) `workers` replicas of it at once, each a single-threaded process stepping
    its own n_steps consecutive batches of the window from the same warm state (the way the
    paper's method itself scales: independent model replicas on disjoint parts of the stream).
    Must run before anything touches the GPU (the replicas are forked)."""
    import multiprocessing as mp
    import numpy as np
    from threadpoolctl import threadpool_limits
    from oracle import tig_oracle as O
    log("building the oracle's neighbour index ...")
    ix = O.NeighbourIndex(g.num_nodes, g.src, g.dst, g.ts)

    def replica(k):
        st = O.OracleState(mem0, lu0)  # (forked: pages the steps touch are copied on write)
        ev = 0
        with threadpool_limits(limits=1):
            for i in range(k * n_steps, (k + 1) * n_steps):
                f, c = batches[i % len(batches)]
                O.step(st, g.src, g.dst, g.ts, g.edge_feat, weights, f, c, negs_np[i % len(batches)],
                       w.num_neighbors, w.num_heads, index=ix, deferred=order == "deferred")
                ev += c
        return ev

    def child(k, q):
        q.put(replica(k))

    st1 = O.OracleState(mem0.copy(), lu0.copy())
    with threadpool_limits(limits=1):
        t0 = time.perf_counter()
        ev1 = 0
        for i in range(n_steps):
            f, c = batches[i]
            O.step(st1, g.src, g.dst, g.ts, g.edge_feat, weights, f, c, negs_np[i], w.num_neighbors,
                   w.num_heads, index=ix, deferred=order == "deferred")
            ev1 += c
        one_s = time.perf_counter() - t0
    del st1
    all_rate, all_s = None, None
    if workers > 1:
        ctx = mp.get_context("fork")
        q = ctx.Queue()
        t0 = time.perf_counter()
        procs = [ctx.Process(target=child, args=(k, q)) for k in range(workers)]
        for p_ in procs:
            p_.start()
        ev_all = sum(q.get() for _ in procs)
        for p_ in procs:
            p_.join()
        all_s = time.perf_counter() - t0
        all_rate = ev_all / all_s
    B = batches[0][1]
    return {"value": round(ev1 / one_s, 1), "unit": "events/s", "cores": 1, "kind": "oracle",
            "sample": f"{n_steps} steps of {B} events of the same window (float64 NumPy oracle, "
                      f"indexed neighbour lookup, index build excluded), {one_s:.1f} s",
            "all_cores": None if all_rate is None else {
                "value": round(all_rate, 1), "cores": workers,
                "sample": f"{workers} single-threaded replicas at once, {n_steps} steps each, {all_s:.1f} s"},
            "cpu_model": cpu_model(), "nproc": os.cpu_count()}


def distinct_queries(g, first, count, nbr_cnt):
    """Rows the embedding kernel computes for the batch: one per distinct (node, t) among the
    sources and destinations (each taken once, with its neighbour count) plus one per negative.
    Returns (rows, filled neighbour slots over those rows)."""
    import numpy as np
    nodes = np.concatenate([g.src[first:first + count], g.dst[first:first + count]]).astype(np.int64)
    times = np.concatenate([g.ts[first:first + count]] * 2)
    _, idx = np.unique(np.stack([nodes.astype(np.float64), times], 1), axis=0, return_index=True)
    rows = len(idx) + count
    slots = int(nbr_cnt[idx].sum()) + int(nbr_cnt[2 * count:].sum())
    return rows, slots


def algorithmic_bytes(w, count, rows_u, slots_u, winners):
    """Bytes the method itself must move per step, by kernel (fp32 state, fp64 times, int32 ids),
    counted over the DISTINCT queries of the batch: rows_u rows with slots_u filled neighbour
    slots (the same (node, t) is looked up and embedded once), `winners` updated nodes."""
    M, F, E, K = w.mem_dim, w.feat_dim, w.emb_dim, w.num_neighbors
    Q = 3 * count
    entries = 2 * count
    src_dst_rows = rows_u - count
    lookup = 4 + 8 + 16 + 4 + 16 * K + 16 * K + 4  # id, time, two offsets, position, window in; slots + count out
    gru = winners * (24 + 8 + (2 * M + F) * 4 + M * 4)  # descriptor, last_update, two memory rows, edge feature in; new row out
    return {
        "k_scatter": 0, "k_select": 0,  # launches of their own only for batches above 4096 events
        # (inside the previous embedding launch in a chronological pass) winners: event reads, one
        # key per entry, descriptors out; queries: event reads and one lookup per distinct pair
        "k_prepare": entries * (4 + 8 + 8) * 2 + winners * (8 + 24) + src_dst_rows * lookup,
        # a launch of its own only when the previous step's closing launch did not run this batch's GRU
        "k_gru": 0,
        # per distinct query: own state row, descriptors; per negative its lookup and one key per
        # filled slot; per filled slot a state row, an edge feature row, reference, event id, time;
        # embedding and the two decoder halves out; per winner: staged row in, memory row and
        # last_update out
        "k_embed": rows_u * (M * 4 + 24) + count * lookup + slots_u * ((M + F) * 4 + 16) + rows_u * 3 * E * 4
        + winners * (24 + 2 * M * 4 + 8),
        # per event: three embedding rows and three decoder halves in, three embedding rows and
        # the scores out; the next batch's GRU; one key read and one reference per filled slot and
        # row of the next batch's distinct source / destination queries
        "k_closing": count * 6 * E * 4 + Q * E * 4 + 2 * count * 4 + gru + (slots_u + rows_u) * 12,
    }


def mfma_flops(w, rows_u, winners, precision):
    """Multiply-adds x 2 the matrix cores execute per launch for the padded tile shapes, and the
    useful part (unpadded, one product per multiply instead of three for split bf16 operands)."""
    def up(x, m):
        return (x + m - 1) // m * m
    kb = 32 if precision == "bf16" else 16
    split = 3 if precision == "bf16" else 1
    M, T, F, E, H = w.mem_dim, w.time_dim, w.feat_dim, w.emb_dim, w.num_heads
    dkv = M + F + T
    dkvp, Mq, Ep, Ek, Ng = up(dkv, kb), up(M, kb), up(E, 16), up(E, kb), up(M, 16)
    Kg, Khn = up(2 * M + T + F, kb), up(M, kb)
    rows16 = up(rows_u, 16)
    win16 = up(winners, 16)
    issued = {
        "k_gru": 2 * win16 * (3 * Ng * Kg + Ng * Khn) * split,
        "k_embed": 2 * rows16 * (H * dkvp * Mq + Ep * (H * dkvp + Mq) + 3 * Ep * Ek) * split,
    }
    useful = {
        "k_gru": 2 * winners * (3 * M * (2 * M + T + F) + M * M),
        "k_embed": 2 * rows_u * (H * dkv * M + E * (H * dkv + M) + 3 * E * E),
    }
    return issued, useful


def train_flops(w, rows, pairs, winners):
    """Multiply-adds x 2 of the contractions of one training step as the kernels run them (attention
    core re-associated: every product over queries, events or winners): forward, backward, weight gradients."""
    M, T, E, F, H = w.mem_dim, w.time_dim, w.emb_dim, w.feat_dim, w.num_heads
    da, dkv, D = M + T, M + F + T, 2 * M + T + F

    def mm(r, n, k):
        return 2.0 * r * n * k
    fwd = mm(rows, da, da) + mm(rows, dkv, da) + mm(rows, da, dkv) + mm(rows, da, da) + mm(rows, E, da + M) + \
        mm(rows, E, E) + mm(pairs, E, 2 * E) + mm(winners, 3 * M, D) + mm(winners, 3 * M, M)
    bwd = mm(pairs, 2 * E, E) + mm(rows, E, E) + mm(rows, da + M, E) + mm(rows, da, da) + mm(rows, dkv, da) + \
        mm(rows, da, dkv) + mm(rows, da, da) + mm(winners, T, 3 * M)
    wgr = mm(pairs, E, 2 * E) + mm(pairs, 1, E) + mm(rows, E, E) + mm(rows, E, da + M) + 2 * mm(rows, da, da) + \
        2 * mm(rows, da, dkv) + mm(winners, 3 * M, D) + mm(winners, 3 * M, M)
    return fwd + bwd + wgr


def bench_train(S, tig, torch, w, g, weights, B, batches, negs, negs_np, mem0, lu0, warm, steps=20, cpu_steps=1,
                rows_per_step=None, winners_per_step=None):
    """Training steps (fp32 masters, deferred message order: a prediction never sees its own event
    through the memory) over consecutive batches of the timed window, lr = 1e-4; beside them the
    training oracle on `cpu_steps` steps of the same window."""
    import numpy as np
    cfg = tig.make_config(w.mem_dim, w.time_dim, w.feat_dim, w.emb_dim, w.num_neighbors, w.num_heads, B, "fp32",
                          "deferred")
    ctx = tig.TigContext(cfg, g.num_nodes, g.src, g.dst, g.ts, g.edge_feat, weights, device="cuda:0")
    ctx.train_attach(weights)
    ctx.state_import(mem0, lu0)
    out = ctx.alloc_outputs(B)
    n_warm = min(3, warm)
    for i in range(n_warm):
        ctx.train_step(batches[i][0], batches[i][1], negs[i], out, 1e-4)
    torch.cuda.synchronize()
    n = min(steps, len(batches) - n_warm)
    t0 = time.perf_counter()
    losses = []
    for i in range(n_warm, n_warm + n):
        losses.append(ctx.train_step(batches[i][0], batches[i][1], negs[i], out, 1e-4).clone())
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ws_bytes = ctx.train_ws.numel()
    ctx.close()
    rep_ = {"steps": n, "ms_per_step": round(dt * 1e3 / n, 3), "events_per_s": round(n * B / dt, 1),
            "order": "deferred", "dtype": "f32", "lr": 1e-4, "workspace_GB": round(ws_bytes / 1e9, 2),
            "loss_first_last": [round(float(losses[0].item()), 5), round(float(losses[-1].item()), 5)]}
    if rows_per_step and winners_per_step:
        fl = train_flops(w, rows_per_step, 2 * B, winners_per_step)
        rep_["contraction_GFLOP_per_step"] = round(fl / 1e9, 2)
        rep_["fp32_mfma_frac_of_peak"] = round(fl / (dt / n) / 1e12 / FP32_MFMA_PEAK_TFLOPS, 4)
    if cpu_steps > 0:
        from threadpoolctl import threadpool_limits
        from oracle import tig_oracle as O
        from oracle import train_oracle as TO
        ix = O.NeighbourIndex(g.num_nodes, g.src, g.dst, g.ts)
        st = O.OracleState(mem0.copy(), lu0.copy())
        Wc = {k: v.copy() for k, v in weights.items()}
        with threadpool_limits(limits=1):
            t0 = time.perf_counter()
            for i in range(cpu_steps):
                TO.train_step(st, g.src, g.dst, g.ts, g.edge_feat, Wc, batches[i][0], batches[i][1], negs_np[i],
                              w.num_neighbors, w.num_heads, 1e-4, index=ix, deferred=True)
            cs = time.perf_counter() - t0
        rep_["oracle_events_per_s"] = round(cpu_steps * B / cs, 1)
        rep_["oracle_sample"] = f"{cpu_steps} training step(s) of {B} events, one core, {cs:.1f} s"
    return rep_


MODULE_INSTANCES = {
    "jodie_like": dict(aggregator="last", updater="rnn", embedding="time_projection"),
    "dyrep_like": dict(aggregator="last", updater="rnn", embedding="identity"),
    "mean_gru_identity": dict(aggregator="mean", updater="gru", embedding="identity"),
    "mean_gru_attention": dict(aggregator="mean", updater="gru", embedding="attention"),
    "two_layer_attention": dict(aggregator="last", updater="gru", embedding="attention", layers=2),
}


def bench_modules(S, tig, torch, w, g, B, batches, negs, negs_np, mem0, lu0, warm, names, steps=50, cpu_steps=1):
    """Other instances of the general architecture (Sec. II-C: mean aggregator, RNN update, identity /
    time-projection embedding) on the timed window, update-first order, fp32: events/s of plain
    tig_step calls, the stage durations from tig_step_profiled, the step's algorithmic bytes against
    the HBM peak, and the instance's oracle on `cpu_steps` steps."""
    import numpy as np
    M, T, F, K_ = w.mem_dim, w.time_dim, w.feat_dim, w.num_neighbors
    report = {}
    for name in names:
        inst = MODULE_INSTANCES[name]
        attn = inst["embedding"] == "attention"
        E = w.emb_dim if attn else M
        Wm = S.make_module_weights(w, inst["updater"], inst["embedding"])
        L2 = S.make_layer2_weights(w) if inst.get("layers", 1) == 2 else None
        cfg = tig.make_config(M, T, F, E, K_, w.num_heads, B, "fp32", "update_first")
        ctx = tig.TigContext(cfg, g.num_nodes, g.src, g.dst, g.ts, g.edge_feat, None, device="cuda:0")
        ctx.modules_attach(Wm, layer2=L2, **inst)
        ctx.state_import(mem0, lu0)
        out = ctx.alloc_outputs(B)
        n_warm = min(5, warm)
        n = min(steps, len(batches) - n_warm)
        for i in range(n_warm):
            ctx.step(batches[i][0], batches[i][1], negs[i], out)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n_warm, n_warm + n):
            ctx.step(batches[i][0], batches[i][1], negs[i], out)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        # stage durations and the byte accounting's counts on a few of the same steps
        ctx.state_import(mem0, lu0)
        insp = ctx.alloc_outputs(B, with_neg=True, inspect=True)
        sums = np.zeros(len(ctx.KERNEL_NAMES))
        n_prof = min(10, n)
        alg = 0.0
        for i in range(n_prof):
            ms = ctx.step_profiled(batches[i][0], batches[i][1], negs[i], insp)
            sums += np.array(ms)
            f, c = batches[i]
            nodes = np.concatenate([g.src[f:f + c], g.dst[f:f + c]])
            n_nodes = int(np.unique(nodes).size)
            msgs = 2 * c if inst["aggregator"] == "mean" else n_nodes
            # applied nodes: own row + last_update in, new row + last_update out; per message partner row + feature row
            by = n_nodes * (8 * M + 16) + msgs * (4 * (M + F) + 16)
            if attn:
                rows_u, slots_u = distinct_queries(g, f, c, insp.nbr_cnt.cpu().numpy())
                by += rows_u * (4 * M + 24) + slots_u * (4 * (M + F) + 16) + 3 * c * 4 * E
                if L2 is not None:
                    # second hop, a lower bound (every neighbour with a full table of its own is not assumed):
                    # per filled slot one more table entry list and the first layer's row written and read back
                    by += slots_u * (16 * K_ + 8 * E)
            else:
                by += 3 * c * (4 * M + 8) + 3 * c * 4 * E      # state rows in, embeddings out
            by += 8 * c
            alg += by
        avg_ms = sums / n_prof
        ctx.close()
        del ctx, out, insp
        torch.cuda.empty_cache()
        r = {"modules": inst, "steps": n, "ms_per_step": round(dt * 1e3 / n, 4), "events_per_s": round(n * B / dt, 1),
             "dtype": "f32", "stage_us": {"selection_and_queries": round(float(avg_ms[:3].sum()) * 1e3, 1),
                                           "update_and_overwrite": round(float(avg_ms[3]) * 1e3, 1),
                                           "embedding_and_decoder": round(float(avg_ms[4]) * 1e3, 1)},
             "alg_bytes_per_step": int(alg / n_prof),
             "hbm_frac": round(alg / n_prof / (dt / n) / 1e9 / HBM_PEAK_GBS, 5)}
        if cpu_steps > 0:
            from threadpoolctl import threadpool_limits
            from oracle import modules_oracle as G
            from oracle import tig_oracle as O
            ix = O.NeighbourIndex(g.num_nodes, g.src, g.dst, g.ts)
            st = O.OracleState(mem0.copy(), lu0.copy())
            mods = G.Modules(inst["aggregator"], inst["updater"], inst["embedding"], None, inst.get("layers", 1), L2)
            with threadpool_limits(limits=1):
                t0 = time.perf_counter()
                for i in range(cpu_steps):
                    G.step(st, g.src, g.dst, g.ts, g.edge_feat, Wm, batches[i][0], batches[i][1], negs_np[i], K_,
                           w.num_heads, mods, index=ix)
                cs = time.perf_counter() - t0
            r["oracle_events_per_s"] = round(cpu_steps * B / cs, 1)
            r["oracle_sample"] = f"{cpu_steps} step(s) of {B} events, one core, {cs:.1f} s"
        report[name] = r
    return report


def bench_sep(g, w, torch, num_parts=8, top_k=0.01, beta=1e-6):
    """The partitioner over the whole stream: centrality kernel (HBM-bound: 16 bytes per event in,
    8 bytes per node out), hub selection, and the sequential edge loop on the host; beside them the
    oracle's edge loop on a bounded prefix of the stream."""
    import numpy as np
    from oracle import sep_oracle as PO
    from paper_2308_14129_amd import sep
    E, N = g.num_events, g.num_nodes
    src_d, dst_d, ts_d = (torch.from_numpy(a).to("cuda:0") for a in (g.src, g.dst, g.ts))
    for _ in range(2):
        cent_d = sep.centrality(src_d, dst_d, ts_d, N, beta)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 5
    e0.record()
    for _ in range(reps):
        cent_d = sep.centrality(src_d, dst_d, ts_d, N, beta)
    e1.record()
    torch.cuda.synchronize()
    cent_ms = e0.elapsed_time(e1) / reps
    n_hubs = int(np.floor(top_k * N))
    t0 = time.perf_counter()
    hubs_d, is_hub_d = sep.top_k(cent_d, n_hubs)
    torch.cuda.synchronize()
    topk_ms = (time.perf_counter() - t0) * 1e3
    cent, is_hub = cent_d.cpu().numpy(), is_hub_d.cpu().numpy()
    cfg = sep.make_config(num_parts, beta, top_k, 1.0, 1e-3)
    t0 = time.perf_counter()
    part, node_parts, part_edges = sep.assign(cfg, g.src, g.dst, N, cent, is_hub)
    assign_s = time.perf_counter() - t0
    n_or = min(E, 200_000)
    t0 = time.perf_counter()
    PO.assign_stream(g.src[:n_or], g.dst[:n_or], N, cent, np.flatnonzero(is_hub), num_parts, 1.0, 1e-3)
    oracle_s = time.perf_counter() - t0
    # sub-graph of one of two combined partitions (parts 0-3 of the 8): order-preserving compaction of
    # the event stream; reads both endpoint arrays twice (count, write), writes the kept event ids
    from paper_2308_14129_amd import pac
    masks_d = torch.from_numpy(node_parts.view(np.int64)).to("cuda:0")
    pac.subgraph(src_d, dst_d, masks_d, 0x0F)
    t0 = time.perf_counter()
    eid_k, _, n_k = pac.subgraph(src_d, dst_d, masks_d, 0x0F)
    torch.cuda.synchronize()
    sub_ms = (time.perf_counter() - t0) * 1e3
    sub_bytes = 16.0 * E + 4.0 * eid_k.numel() + 12.0 * N
    cent_bytes = 16.0 * E + 16.0 * N  # events in; node array cleared and written
    bits = np.unpackbits(node_parts.view(np.uint8).reshape(-1, 8), axis=1).sum(axis=1)
    return {"num_parts": num_parts, "top_k": top_k, "beta": beta,
            "centrality_ms": round(cent_ms, 3), "centrality_GBps": round(cent_bytes / cent_ms / 1e6, 1),
            "centrality_frac_of_hbm_peak": round(cent_bytes / cent_ms / 1e6 / HBM_PEAK_GBS, 4),
            "top_k_ms": round(topk_ms, 2),
            "assign_edges_per_s": round(E / assign_s, 1), "assign_s": round(assign_s, 2),
            "oracle_assign_edges_per_s": round(n_or / oracle_s, 1), "oracle_sample_edges": n_or,
            "subgraph_ms": round(sub_ms, 3), "subgraph_GBps": round(sub_bytes / sub_ms / 1e6, 1),
            "subgraph_events": int(eid_k.numel()), "subgraph_nodes": n_k,
            "edge_cut": round(float(np.mean(part < 0)), 7), "shared_nodes": int((bits > 1).sum()),
            "part_edges_min_max": [int(part_edges.min()), int(part_edges.max())]}


def derive_partition(S, torch, w, scale, n_hubs, num_parts=None, beta=1e-6):
    """One GPU's partition DERIVED instead of postulated: a parent stream of `scale` times the
    workload's events over `scale` times its owned ids is cut by the streaming edge partitioner
    (Sec. II-B, Alg. 1) into `num_parts` partitions (default: `scale`) with the `n_hubs` most central
    nodes replicated; partition 0's sub-graph (Sec. II-C: the events between its members, shared hubs
    included, local ids) becomes the workload the step is timed on.  Returns (workload, graph, report).
    With rank-frequency Zipf endpoints most events run between two hubs, and the shared hubs are
    members of every partition: a partition's sub-graph then holds nearly the whole parent stream."""
    num_parts = num_parts or scale
    import dataclasses
    import numpy as np
    from paper_2308_14129_amd import pac, sep
    owned = w.n_src - n_hubs
    parent = dataclasses.replace(w, name=w.name + "_parent", n_src=scale * owned + n_hubs, num_events=scale * w.num_events)
    t0 = time.time()
    gp = S.make_graph(parent, with_features=False)
    N, E = gp.num_nodes, gp.num_events
    log(f"parent stream: {N} ids, {E} events, generated in {time.time() - t0:.1f} s")
    src_d, dst_d, ts_d = (torch.from_numpy(a).to("cuda:0") for a in (gp.src, gp.dst, gp.ts))
    top_k = n_hubs / N
    cent_d = sep.centrality(src_d, dst_d, ts_d, N, beta)
    hubs_d, is_hub_d = sep.top_k(cent_d, n_hubs)
    torch.cuda.synchronize()
    cent, is_hub = cent_d.cpu().numpy(), is_hub_d.cpu().numpy()
    cfg = sep.make_config(num_parts, beta, top_k, 1.0, 1e-3)
    t0 = time.perf_counter()
    part, node_parts, part_edges = sep.assign(cfg, gp.src, gp.dst, N, cent, is_hub)
    assign_s = time.perf_counter() - t0
    log(f"edge loop: {assign_s:.1f} s ({E / assign_s / 1e6:.1f} M edges/s)")
    copies = np.unpackbits(node_parts.view(np.uint8).reshape(-1, 8), axis=1).sum(axis=1)
    placed = copies > 0
    n_shared = int((copies > 1).sum())
    rf = (n_shared * num_parts + (int(placed.sum()) - n_shared)) / max(1, int(placed.sum()))  # a shared node is listed in every partition
    masks_d = torch.from_numpy(node_parts.view(np.int64)).to("cuda:0")
    t0 = time.perf_counter()
    eid_k, local_d, n_k = pac.subgraph(src_d, dst_d, masks_d, 1)
    dummy = torch.empty((E, 1), dtype=torch.float32, device="cuda:0")  # the parent has no feature rows: the sub-graph draws its own
    s_k, d_k, t_k, _ = pac.gather(src_d, dst_d, ts_d, dummy, eid_k, local_d)
    torch.cuda.synchronize()
    sub_s = time.perf_counter() - t0
    n_e = int(eid_k.numel())
    src_k, dst_k, ts_k = s_k.cpu().numpy(), d_k.cpu().numpy(), t_k.cpu().numpy()
    hubs_in = int(is_hub_d[(local_d >= 0)].sum().item())
    del src_d, dst_d, ts_d, dummy, eid_k, local_d, s_k, d_k, t_k, masks_d, cent_d, hubs_d, is_hub_d
    torch.cuda.empty_cache()
    name = w.name.replace("gpu_partition", "derived_partition") if "gpu_partition" in w.name else w.name + "_derived_partition"
    ws = dataclasses.replace(w, name=name, n_src=n_k, num_events=n_e)
    g = S.Graph(n_k, src_k, dst_k, ts_k, S.make_edge_feat(ws, n_e))
    report = {"parent_nodes": N, "parent_events": E, "num_parts": num_parts, "hubs": n_hubs, "top_k": round(top_k, 6),
              "beta": beta, "assign_s": round(assign_s, 1), "assign_edges_per_s": round(E / assign_s, 1),
              "edge_cut": round(float(np.mean(part < 0)), 8), "nodes_placed": int(placed.sum()),
              "shared_nodes": n_shared, "replication_factor": round(rf, 5),
              # Theorem 1 over the nodes that occur: the hubs are the fraction k' of them, RF <= k'|P| + (1 - k')
              "theorem_1_bound": round((n_hubs * num_parts + int(placed.sum()) - n_hubs) / max(1, int(placed.sum())), 5),
              "part_edges_min_max": [int(part_edges.min()), int(part_edges.max())],
              "subgraph_and_gather_s": round(sub_s, 3), "partition_nodes": n_k, "partition_hubs": hubs_in,
              "partition_events": n_e}
    log(f"partition 0: {n_k} nodes ({hubs_in} hubs), {n_e} events; RF {rf:.4f} <= {report['theorem_1_bound']}")
    return ws, g, report


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c5_gpu_partition")
    ap.add_argument("--precision", default=None, choices=[None, "fp32", "bf16"])
    ap.add_argument("--window", type=float, default=0.5, help="start of the timed window, fraction of the stream")
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-steps", type=int, default=2)
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run three plain 256 MiB device copies (known HBM traffic) so that a "
                         "rocprofv3 --pmc run of this command can scale FETCH_SIZE / WRITE_SIZE")
    ap.add_argument("--order", default="update_first", choices=["update_first", "deferred"],
                    help="message order of the step: apply this batch's messages before embedding "
                         "(default, the headline configuration) or the previous batch's (training order)")
    ap.add_argument("--ceilings", action="store_true",
                    help="also time a plain 1 GiB device copy (read + write) and report the measured "
                         "HBM bandwidth of this GPU beside the published peak")
    ap.add_argument("--sep", action="store_true",
                    help="also run the streaming edge partitioner (Sec. II-B) over the workload's whole event "
                         "stream (8 partitions, 1 %% hubs) and report its stages in a \"sep\" object")
    ap.add_argument("--train", action="store_true", help="(the default; kept for older command lines)")
    ap.add_argument("--no-train", action="store_true",
                    help="skip the training steps (forward, BCE loss, backward, SGD; fp32, deferred message order) "
                         "that are otherwise timed on the same window and reported in a \"train\" object")
    ap.add_argument("--modules", default=None,
                    help="also time other instances of the general architecture (comma-separated names of "
                         "MODULE_INSTANCES, or 'all') on the same window and report them in a \"modules\" object")
    ap.add_argument("--derive", action="store_true",
                    help="time the step on a partition DERIVED by the streaming edge partitioner from a parent "
                         "stream of --derive-scale times the workload's events (partition 0 of --derive-parts), "
                         "instead of on the workload as postulated; reported in a \"derived\" object (no CPU baseline)")
    ap.add_argument("--derive-scale", type=int, default=1)
    ap.add_argument("--derive-parts", type=int, default=4)
    ap.add_argument("--derive-hubs", type=int, default=100_000)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import tig_synth as S
    from paper_2308_14129_amd import tig

    w = S.WORKLOADS[args.workload]
    precision = args.precision or w.precision
    B = args.batch or w.batch_size
    K, W_ = args.steps, args.warmup
    t0 = time.time()
    log(f"generating {w.name}: {w.num_nodes} nodes, {w.num_events} events ...")
    derived = None
    if args.derive:
        if w.bipartite or not torch.cuda.is_available():
            print("bench.py: --derive needs a GPU and a workload with one id space", file=sys.stderr)
            sys.exit(1)
        args.no_cpu_baseline = True  # (the oracle's replicas are forked, which must happen before the GPU is touched)
        w, g, derived = derive_partition(S, torch, w, args.derive_scale, args.derive_hubs, args.derive_parts)
    else:
        g = S.make_graph(w)
    weights = S.make_weights(w)
    log(f"generated in {time.time() - t0:.1f} s")

    total_steps = W_ + K
    first = int(w.num_events * args.window) // B * B
    if first + total_steps * B > w.num_events:
        first = max(0, (w.num_events - total_steps * B) // B * B)
    batches = list(S.batches(w.num_events, B, first=first, stop=first + total_steps * B))
    assert len(batches) == total_steps, "workload too short for the requested steps"

    mem0, lu0 = S.make_warm_state(w, g, first)
    negs_np = np.stack([S.make_negatives(w, g, f, c) for f, c in batches])

    # ---- CPU baseline first (its replicas are forked, which must happen before the GPU is touched):
    # the oracle, as it stands, on a bounded sample of the timed window
    cpu = None
    if not args.no_cpu_baseline:
        workers = max(1, min(16, os.cpu_count() or 1, len(batches[W_:]) // max(1, args.cpu_steps)))
        cpu = oracle_baseline(g, w, weights, batches[W_:], negs_np[W_:], mem0, lu0, args.order,
                              max(1, min(args.cpu_steps, K)), workers)
        log(f"oracle: {cpu['value']} events/s on one core, "
            f"{cpu['all_cores']['value'] if cpu['all_cores'] else '-'} on {workers}")

    tig.load_library()  # fails loudly if libtig.so is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    cfg = tig.make_config(w.mem_dim, w.time_dim, w.feat_dim, w.emb_dim, w.num_neighbors, w.num_heads, B,
                          precision, args.order)
    t0 = time.time()
    ctx = tig.TigContext(cfg, g.num_nodes, g.src, g.dst, g.ts, g.edge_feat, weights, device="cuda:0")
    torch.cuda.synchronize()
    log(f"tig_init in {time.time() - t0:.1f} s (persistent {ctx.persistent_bytes / 1e9:.2f} GB, "
        f"scratch {ctx.scratch_bytes / 1e9:.2f} GB)")

    negs = torch.from_numpy(negs_np).to("cuda:0")
    out = ctx.alloc_outputs(B, with_neg=True, inspect=False)
    torch.cuda.synchronize()

    def run(lo, hi):
        for i in range(lo, hi):
            ctx.step(batches[i][0], batches[i][1], negs[i], out)

    # ---- throughput: W warm-up steps, then exactly K timed steps ---------------------------------
    ctx.state_import(mem0, lu0)
    run(0, W_)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_start = time.perf_counter()
    ev0.record()
    run(W_, total_steps)
    ev1.record()
    torch.cuda.synchronize()
    wall_s = time.perf_counter() - t_start
    gpu_ms = ev0.elapsed_time(ev1)
    events = sum(c for _, c in batches[W_:])
    ms_per_step = wall_s * 1e3 / K
    value = events / wall_s

    # ---- per-kernel durations: HIP events on the context's stream around every kernel of the SAME
    # launch sequence the timed region ran (same batches, prepared ahead in the same way, no
    # inspection outputs).  The byte accounting needs the neighbour counts and winner flags of
    # those batches: a pass of its own, before, asks for them. ---------------------------------
    names = ctx.KERNEL_NAMES
    n_prof = min(K, 50)
    ctx.state_import(mem0, lu0)
    run(0, W_)
    insp = ctx.alloc_outputs(B, with_neg=True, inspect=True)
    byte_sums = {n: 0.0 for n in names}
    rows_sum = slots_sum = win_sum = 0
    for i in range(W_, W_ + n_prof):
        ctx.step(batches[i][0], batches[i][1], negs[i], insp)
        torch.cuda.synchronize()
        rows_u, slots_u = distinct_queries(g, batches[i][0], batches[i][1], insp.nbr_cnt.cpu().numpy())
        winners = int(insp.is_winner.sum().item())
        rows_sum, slots_sum, win_sum = rows_sum + rows_u, slots_sum + slots_u, win_sum + winners
        for n, v in algorithmic_bytes(w, batches[i][1], rows_u, slots_u, winners).items():
            byte_sums[n] += v
    del insp
    ctx.state_import(mem0, lu0)
    run(0, W_)
    torch.cuda.synchronize()
    sums = np.zeros(len(names))
    launches_prof = set()
    for i in range(W_, W_ + n_prof):
        ms = ctx.step_profiled(batches[i][0], batches[i][1], negs[i], out)
        launches_prof.add(ctx.launch_info()["kernels_per_step"])
        sums += np.array(ms)
    avg_ms = sums / n_prof
    dom = int(np.argmax(avg_ms))
    dom_name = names[dom]
    dom_bytes = byte_sums[dom_name] / n_prof
    achieved = dom_bytes / (avg_ms[dom] * 1e-3) / 1e9
    stages = {n: {"avg_us": round(float(avg_ms[i]) * 1e3, 2),
                  "alg_bytes": int(byte_sums[n] / n_prof),
                  "GBps": round(byte_sums[n] / n_prof / max(float(avg_ms[i]), 1e-9) / 1e6, 1)}
              for i, n in enumerate(names) if avg_ms[i] > 1e-4}   # (a launch the steps did not need reads 0)
    figs = profile_figures("counters", w.name, precision, B)
    trace = profile_figures("step_kernels", w.name, precision, B)
    traffic = float(figs["k_embed_hbm_bytes_per_launch"]) if dom_name == "k_embed" and \
        "k_embed_hbm_bytes_per_launch" in figs else None
    roofline = {"bound": "hbm", "kernel": dom_name, "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 5), "traffic": traffic,
                "avg_kernel_us": round(float(avg_ms[dom]) * 1e3, 2), "alg_bytes_per_launch": int(dom_bytes),
                "profiled_steps": n_prof, "kernels_per_profiled_step": sorted(launches_prof),
                "distinct_query_rows": round(rows_sum / n_prof, 1), "queries": 3 * B,
                "winners": round(win_sum / n_prof, 1)}
    if dom_name + "_trace_avg_us" in trace:
        # the same kernel's average duration in the committed rocprofv3 kernel trace (the event pair
        # around a launch reads a few microseconds high on this machine)
        t_us = float(trace[dom_name + "_trace_avg_us"])
        roofline["trace_avg_kernel_us"] = t_us
        roofline["trace_frac"] = round(dom_bytes / (t_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 5)
    if traffic:
        roofline["traffic_frac_of_peak"] = round(traffic / (float(avg_ms[dom]) * 1e-3) / 1e9 / HBM_PEAK_GBS, 5)
    issued, useful = mfma_flops(w, rows_sum / n_prof, win_sum / n_prof, precision)
    peak_tf = BF16_PEAK_TFLOPS if precision == "bf16" else FP32_MFMA_PEAK_TFLOPS
    mfma = {}
    for n in ("k_gru", "k_embed"):
        # (in a chronological pass the GRU runs inside the closing launch of the step before)
        t_s = float(avg_ms[names.index("k_closing" if n == "k_gru" else n)]) * 1e-3
        mfma[n] = {"issued_GFLOP": round(issued[n] / 1e9, 3), "useful_GFLOP": round(useful[n] / 1e9, 3),
                   "issued_frac_of_peak": round(issued[n] / t_s / 1e12 / peak_tf, 5),
                   "useful_frac_of_peak": round(useful[n] / t_s / 1e12 / peak_tf, 5)}
    mfma["peak_TFLOPs"] = peak_tf
    for k in ("k_embed_mfma_busy_frac", "k_gru_mfma_busy_frac", "k_embed_mfma_flop_per_launch",
              "k_gru_mfma_flop_per_launch"):
        if k in figs:
            mfma[k + "_counter"] = float(figs[k])

    if args.pmc_calibration:
        n = 256 << 20
        src_buf = torch.full((n,), 1, dtype=torch.uint8, device="cuda:0")
        dst_buf = torch.empty_like(src_buf)
        for _ in range(3):
            dst_buf.copy_(src_buf)   # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src_buf, dst_buf

    measured_copy_gbs = None
    if args.ceilings:
        n = 1 << 30
        src_buf = torch.full((n,), 1, dtype=torch.uint8, device="cuda:0")
        dst_buf = torch.empty_like(src_buf)
        for _ in range(3):
            dst_buf.copy_(src_buf)
        torch.cuda.synchronize()
        c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        c0.record()
        for _ in range(10):
            dst_buf.copy_(src_buf)
        c1.record()
        torch.cuda.synchronize()
        measured_copy_gbs = round(10 * 2 * n / (c0.elapsed_time(c1) * 1e-3) / 1e9, 1)  # bytes read + written
        del src_buf, dst_buf
        roofline["measured_copy_GBps"] = measured_copy_gbs

    info = ctx.launch_info()
    train_report = None
    if not args.no_train:
        ctx.close()
        del ctx
        torch.cuda.empty_cache()
        train_report = bench_train(S, tig, torch, w, g, weights, B, batches, negs, negs_np, mem0, lu0, W_,
                                   cpu_steps=0 if args.no_cpu_baseline else 1, rows_per_step=rows_sum / n_prof,
                                   winners_per_step=win_sum / n_prof)
        ctx = None

    modules_report = None
    if args.modules:
        names_m = list(MODULE_INSTANCES) if args.modules == "all" else args.modules.split(",")
        if ctx is not None:
            ctx.close()
            ctx = None
            torch.cuda.empty_cache()
        modules_report = bench_modules(S, tig, torch, w, g, B, batches, negs, negs_np, mem0, lu0, W_, names_m,
                                       cpu_steps=0 if args.no_cpu_baseline else 1)

    sep_report = None
    if args.sep:
        sep_report = bench_sep(g, w, torch)

    line = {
        "metric": "events/sec per TGN batch step (1 MI355X)",
        "value": round(value, 1),
        "unit": "events/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W_,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if precision == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "num_nodes": w.num_nodes, "num_events": w.num_events,
                   "batch": B, "K": w.num_neighbors, "heads": w.num_heads, "mem_dim": w.mem_dim,
                   "time_dim": w.time_dim, "feat_dim": w.feat_dim, "emb_dim": w.emb_dim,
                   "precision": "bf16 hi/lo split MFMA operands, fp32 accumulate" if precision == "bf16"
                   else "fp32 MFMA", "window_first_eid": first, "queries_per_event": 3,
                   "message_order": args.order},
        "gpu_ms_per_step_events": round(gpu_ms / K, 5),
        "kernels_per_step": info["kernels_per_step"],
        "roofline": roofline,
        "mfma_util": mfma,
        "stages": stages,
        "cpu_baseline": cpu,
    }
    if sep_report is not None:
        line["sep"] = sep_report
    if train_report is not None:
        line["train"] = train_report
    if modules_report is not None:
        line["modules"] = modules_report
    if derived is not None:
        line["derived"] = derived
    if ctx is not None:
        ctx.close()
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
