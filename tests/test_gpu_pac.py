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
