"""Epoch machinery on the GPU against the oracle (Sec. II-C "Distributed Parallel Training",
Alg. 2): sub-graphs of combined partitions bit for bit, an epoch over several resident partitions
(state within the step's tolerance, last_update bit for bit), shared-node synchronisation."""
import numpy as np
import pytest

import tig_synth as S
from oracle import pac_oracle as E
from oracle import sep_oracle as P
from oracle import tig_oracle as O
from tests.parity import gate
from tests.test_gpu_parity import make_ctx

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


@pytest.fixture(scope="module")
def cut():
    """C1 cut into 8 small parts by the partitioner's oracle."""
    w = S.WORKLOADS["c1_tiny"]
    g = S.make_graph(w)
    r = P.partition(g.src, g.dst, g.ts, g.num_nodes, 8, beta=1e-5, k_frac=0.02, lam=1.0, eps=1e-3)
    masks = np.array([sum(1 << p for p in a) for a in r["A"]], dtype=np.uint64)
    return w, g, S.make_weights(w), masks


def test_subgraphs_of_combined_partitions(cut):
    from paper_2308_14129_amd import pac
    w, g, W, masks = cut
    order = np.random.default_rng(5).permutation(8)
    for gm in pac.combine(order, 4) + [1, 0xFF, 0]:
        print(f"[pac] subgraph group {gm:#x}", flush=True)
        ref_eids, ref_local, ref_n = E.subgraph(g.src, g.dst, masks, 8, gm)
        eid, local, n = pac.subgraph(dev(g.src), dev(g.dst), dev(masks.view(np.int64)), gm)
        assert n == ref_n
        assert np.array_equal(eid.cpu().numpy(), ref_eids)
        assert np.array_equal(local.cpu().numpy(), ref_local)
        if len(ref_eids):
            s, d, t, f = pac.gather(dev(g.src), dev(g.dst), dev(g.ts), dev(g.edge_feat), eid, local)
            assert np.array_equal(s.cpu().numpy(), ref_local[g.src[ref_eids]])
            assert np.array_equal(d.cpu().numpy(), ref_local[g.dst[ref_eids]])
            assert np.array_equal(t.cpu().numpy(), g.ts[ref_eids])
            assert np.array_equal(f.cpu().numpy(), g.edge_feat[ref_eids])


def _resident_parts(cut, groups, batch, deferred=False):
    """Sub-graphs of the groups, built by the library on the device; contexts and oracle twins over them."""
    import torch
    from paper_2308_14129_amd import pac
    w, g, W, masks = cut
    src_d, dst_d, ts_d, f_d = dev(g.src), dev(g.dst), dev(g.ts), dev(g.edge_feat)
    masks_d = dev(masks.view(np.int64))
    gpu, ref, locals_ = [], [], []
    for gm in groups:
        eid, local, n = pac.subgraph(src_d, dst_d, masks_d, gm)
        s, d, t, f = pac.gather(src_d, dst_d, ts_d, f_d, eid, local)
        torch.cuda.synchronize()
        s_h, d_h, t_h, f_h = s.cpu().numpy(), d.cpu().numpy(), t.cpu().numpy(), f.cpu().numpy()
        sub = type("G", (), {"num_nodes": n, "src": s_h, "dst": d_h, "ts": t_h, "edge_feat": f_h})
        ctx = make_ctx(w, sub, W, "fp32", batch, "deferred" if deferred else "update_first")
        neg = ((np.arange(len(s_h)) * 7919 + 13) % n).astype(np.int32)
        neg = np.where(neg == s_h, (neg + 1) % n, neg).astype(np.int32)
        gpu.append({"ctx": ctx, "batch": batch, "num_events": len(s_h), "neg": dev(neg),
                    "backup_mem": torch.zeros((n, w.mem_dim), dtype=torch.float32, device="cuda:0"),
                    "backup_lu": torch.zeros(n, dtype=torch.float64, device="cuda:0"),
                    "out": ctx.alloc_outputs(batch)})
        ref.append({"num_nodes": n, "mem_dim": w.mem_dim, "src": s_h, "dst": d_h, "ts": t_h, "edge_feat": f_h,
                    "W": W, "batch": batch, "neg": neg})
        locals_.append(local.cpu().numpy())
    return gpu, ref, locals_


@pytest.mark.parametrize("deferred", [False, True])
def test_epoch_over_resident_partitions(cut, deferred):
    import torch
    from paper_2308_14129_amd import pac
    w = cut[0]
    groups = pac.combine(np.random.default_rng(9).permutation(8), 4)[:3]   # three of the four partitions
    gpu, ref, _ = _resident_parts(cut, groups, batch=150, deferred=deferred)
    n_batches = [(p["num_events"] + 149) // 150 for p in gpu]
    print(f"[pac] epoch: batches per partition {n_batches}", flush=True)
    assert len(set(n_batches)) > 1                                          # some partition has to loop
    final, trace, ref_steps = E.epoch(ref, w.num_neighbors, w.num_heads, deferred=deferred)
    steps = pac.epoch(gpu)
    torch.cuda.synchronize()
    assert steps == ref_steps == max(n_batches)
    for k, p in enumerate(gpu):
        mem, lu = p["ctx"].state_export()
        assert np.array_equal(lu, final[k].last_update)
        gate(mem, final[k].mem, 1e-4, f"memory of partition {k}")
        assert np.array_equal(p["backup_lu"].cpu().numpy(), final[k].last_update)
        p["ctx"].close()


@pytest.mark.parametrize("mode", ["latest", "mean"])
def test_shared_node_synchronisation(cut, mode):
    import torch
    from paper_2308_14129_amd import pac
    w, g, W, masks = cut
    groups = pac.combine(np.arange(8), 4)
    gpu, ref, locals_ = _resident_parts(cut, groups, batch=200)
    bits = np.array([bin(int(m)).count("1") for m in masks])
    shared = np.flatnonzero(bits > 1)
    assert len(shared) > 0
    ids = [loc[shared].astype(np.int32) for loc in locals_]
    assert all((i >= 0).all() for i in ids)                                  # shared nodes reside everywhere
    # a few steps on every partition, so that the replicas differ; then the exchange
    states = []
    for p, r in zip(gpu, ref):
        st = O.OracleState.zeros(r["num_nodes"], r["mem_dim"])
        for first in (0, 200, 400):
            p["ctx"].step(first, 200, p["neg"][first:first + 200], p["out"])
            O.step(st, r["src"], r["dst"], r["ts"], r["edge_feat"], W, first, 200, r["neg"][first:first + 200],
                   w.num_neighbors, w.num_heads)
        states.append(st)
    torch.cuda.synchronize()
    # both sides start the exchange from the GPU's own state, so the exchange itself is compared exactly
    for p, st in zip(gpu, states):
        mem, lu = p["ctx"].state_export()
        assert np.array_equal(lu, st.last_update)
        gate(mem, st.mem, 1e-4, "memory before the exchange")
        st.mem[:] = mem
    E.sync_shared(states, ids, mode)
    pac.sync_shared([p["ctx"] for p in gpu], [dev(i) for i in ids], mode)
    torch.cuda.synchronize()
    for p, st in zip(gpu, states):
        mem, lu = p["ctx"].state_export()
        assert np.array_equal(lu, st.last_update) and np.array_equal(mem, st.mem)
    # the step after the exchange reads the exchanged memory (nothing staged before it is reused)
    for p, r, st in zip(gpu, ref, states):
        o = p["ctx"].alloc_outputs(200)
        p["ctx"].step(600, 200, p["neg"][600:800], o)
        want = O.step(st, r["src"], r["dst"], r["ts"], r["edge_feat"], W, 600, 200, r["neg"][600:800],
                      w.num_neighbors, w.num_heads)
        torch.cuda.synchronize()
        gate(o.emb.cpu().numpy(), want["emb"], 1e-4, "emb after the exchange")
        p["ctx"].close()


def test_partition_derived_from_a_parent_stream_is_a_valid_workload():
    """bench.py --derive: a parent stream cut by the partitioner into four parts, part 0 extracted on the
    device with local ids.  The result must be a well-formed chronological stream over its own ids, every
    event an event of the parent between two members, within Theorem 1's replication bound."""
    import torch
    import bench
    w = S.WORKLOADS["c1_tiny"]
    ws, g, rep = bench.derive_partition(S, torch, w, 4, 50)
    assert g.num_nodes == rep["partition_nodes"] == ws.num_nodes and g.num_events == rep["partition_events"] == ws.num_events
    assert rep["parent_events"] == 4 * w.num_events and rep["parent_nodes"] == 4 * (w.num_nodes - 50) + 50
    assert 0 < g.num_events < rep["parent_events"]
    assert np.all(np.diff(g.ts) >= 0) and np.all(g.src != g.dst)
    assert g.src.min() >= 0 and g.dst.min() >= 0 and max(g.src.max(), g.dst.max()) < g.num_nodes
    assert rep["replication_factor"] <= rep["theorem_1_bound"] + 1e-12
    assert rep["partition_hubs"] <= 50 and g.edge_feat.shape == (g.num_events, w.feat_dim)
    # the same cut by the oracle's own stream loop keeps the same events (when no decision was near a tie)
    import dataclasses
    parent = dataclasses.replace(w, n_src=rep["parent_nodes"], num_events=rep["parent_events"])
    gp = S.make_graph(parent, with_features=False)
    cent = P.centrality(gp.src, gp.dst, gp.ts, gp.num_nodes, rep["beta"])
    order = sorted(range(len(cent)), key=lambda i: (-cent[i], i))
    gap = cent[order[49]] - cent[order[50]]
    _, A, _, margin = P.assign_stream(gp.src, gp.dst, gp.num_nodes, cent, sorted(order[:50]), 4, 1.0, 1e-3)
    if margin > 1e-9 and gap > 1e-9:
        members = np.array([len(a) > 1 or a == {0} for a in A], dtype=bool)
        keep = members[gp.src] & members[gp.dst]
        assert int(keep.sum()) == g.num_events and int(members.sum()) == g.num_nodes
        np.testing.assert_array_equal(g.ts, gp.ts[keep])
        np.testing.assert_array_equal(g.src, (np.cumsum(members) - 1)[gp.src[keep]])


def test_gather_beyond_the_thread_limit_of_one_dispatch():
    """One wavefront per event would need more than 2^32 threads above 67 M events: the gather strides."""
    import torch
    from paper_2308_14129_amd import pac
    n, N = 70_000_000, 1000
    dev = "cuda:0"
    src = (torch.arange(n, device=dev, dtype=torch.int64) % N).to(torch.int32)
    dst = ((torch.arange(n, device=dev, dtype=torch.int64) * 7 + 1) % N).to(torch.int32)
    ts = torch.arange(n, device=dev, dtype=torch.float64)
    feat = torch.arange(n, device=dev, dtype=torch.float32).reshape(n, 1)
    eid = torch.arange(n - 1, -1, -1, device=dev, dtype=torch.int32)      # reversed: every row moves
    local = torch.arange(N, device=dev, dtype=torch.int32) + 5
    s, d, t, f = pac.gather(src, dst, ts, feat, eid, local)
    torch.cuda.synchronize()
    for w in (0, 1, 67_108_863, 67_108_864, n - 2, n - 1):
        e = n - 1 - w
        assert int(s[w]) == e % N + 5 and int(d[w]) == (e * 7 + 1) % N + 5
        assert float(t[w]) == float(e) and float(f[w, 0]) == float(np.float32(e))
    assert bool((t == torch.arange(n - 1, -1, -1, device=dev, dtype=torch.float64)).all())
