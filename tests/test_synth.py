"""Properties of the seeded workload generator (inputs only)."""
import numpy as np

import tig_synth as S


def test_c1_graph_properties_and_determinism():
    w = S.WORKLOADS["c1_tiny"]
    a, b = S.make_graph(w), S.make_graph(w)
    for x, y in ((a.src, b.src), (a.dst, b.dst), (a.ts, b.ts), (a.edge_feat, b.edge_feat)):
        assert np.array_equal(x, y)
    assert a.src.dtype == np.int32 and a.ts.dtype == np.float64 and a.edge_feat.dtype == np.float32
    assert a.num_events == 10_000 and a.edge_feat.shape == (10_000, 16)
    assert np.all(np.diff(a.ts) >= 0) and a.ts[0] >= 0 and a.ts[-1] < 1e5
    assert np.all(a.src != a.dst)
    assert a.src.min() >= 0 and max(a.src.max(), a.dst.max()) < 1000
    # rank-frequency Zipf(1.2) over 1000 ids: the top id draws about 23 % of the endpoints
    share = np.bincount(np.concatenate([a.src, a.dst]), minlength=1000)[0] / 20_000
    assert 0.15 < share < 0.30
    assert abs(a.edge_feat.mean()) < 0.02 and abs(a.edge_feat.std() - 1) < 0.02


def test_bipartite_ids_and_integer_seconds():
    w = S.WORKLOADS["c2_bipartite_medium"].scaled(num_events=30_000)
    g = S.make_graph(w, with_features=False)
    assert g.src.max() < w.n_src and g.dst.min() >= w.n_src and g.dst.max() < w.num_nodes
    assert np.array_equal(g.ts, np.floor(g.ts)) and g.ts[-1] < w.span
    assert np.all(np.diff(g.ts) >= 0)


def test_thread_count_does_not_change_timestamps():
    import os
    import subprocess
    import sys
    code = ("import tig_synth as S, hashlib;"
            "g=S.make_graph(S.WORKLOADS['c3_bipartite_dense'].scaled(num_events=300000),False);"
            "print(hashlib.sha1(g.ts.tobytes()+g.src.tobytes()).hexdigest())")
    outs = []
    for nt in ("1", "5"):
        env = dict(os.environ, OMP_NUM_THREADS=nt)
        outs.append(subprocess.run([sys.executable, "-c", code], env=env, capture_output=True,
                                   text=True, check=True,
                                   cwd=os.path.dirname(os.path.dirname(os.path.abspath(__file__)))).stdout)
    assert outs[0] == outs[1] and len(outs[0]) > 20


def test_negatives_and_warm_state():
    w = S.WORKLOADS["c1_tiny"]
    g = S.make_graph(w)
    neg = S.make_negatives(w, g, 500, 200)
    assert np.all(neg != g.src[500:700]) and neg.min() >= 0 and neg.max() < 1000
    assert np.array_equal(neg, S.make_negatives(w, g, 500, 200))
    wb = S.WORKLOADS["c2_bipartite_medium"].scaled(num_events=5000)
    gb = S.make_graph(wb, with_features=False)
    nb = S.make_negatives(wb, gb, 0, 1000)
    assert nb.min() >= wb.n_src and nb.max() < wb.num_nodes
    mem, lu = S.make_warm_state(w, g, 3000)
    seen = np.zeros(1000, dtype=bool)
    seen[g.src[:3000]] = True
    seen[g.dst[:3000]] = True
    assert not mem[~seen].any() and not lu[~seen].any()
    assert np.all(np.abs(mem[seen]) <= 0.5) and mem[seen].std() > 0.2
    for u in np.flatnonzero(seen)[:50]:
        last = np.flatnonzero((g.src[:3000] == u) | (g.dst[:3000] == u)).max()
        assert lu[u] == g.ts[last]


def test_weights_shapes_and_param_counts():
    for name, want in (("c1_tiny", 29_217), ("c2_bipartite_medium", 873_233),
                       ("c4_million_node", 353_201), ("c5_gpu_partition", 347_601)):
        w = S.WORKLOADS[name]
        W = S.make_weights(w)
        assert S.num_params(W) == want
        lim = np.sqrt(6.0 / (W["W_i"].shape[0] + W["W_i"].shape[1]))
        assert np.abs(W["W_i"]).max() <= lim and np.abs(W["W_i"]).max() > 0.9 * lim
        assert W["time_w"][0] == 1.0 and abs(W["time_w"][-1] - 1e-9) < 1e-15
        assert np.abs(W["b_i"]).max() <= 0.1
