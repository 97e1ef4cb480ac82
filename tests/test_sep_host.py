"""The host stage of the partitioner (tig_sep_assign: the sequential edge loop of Alg. 1) against
the oracle, bit for bit, on the oracle's own centralities and hubs.  No GPU needed."""
import json
import os

import numpy as np
import pytest

import tig_synth as S
from oracle import sep_oracle as P

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "sep_hand_stream.json")


@pytest.fixture(scope="module")
def sep():
    from paper_2308_14129_amd import sep, tig
    if not os.path.exists(tig.LIB_PATH):
        from paper_2308_14129_amd import build
        build.build()
    return sep


def masks(A):
    return np.array([sum(1 << p for p in a) for a in A], dtype=np.uint64)


def test_hand_worked_stream(sep):
    g = json.load(open(GOLDEN))
    is_hub = np.zeros(g["num_nodes"], dtype=np.uint8)
    is_hub[g["hubs"]] = 1
    cfg = sep.make_config(g["num_parts"], 0.0, 0.0, g["lambda"], g["epsilon"])
    part, node_parts, sizes = sep.assign(cfg, g["src"], g["dst"], g["num_nodes"], g["cent"], is_hub)
    assert part.tolist() == g["edge_part"]
    assert node_parts.tolist() == masks(g["A"]).tolist()
    assert sizes.tolist() == g["sizes"]
    parts, shared = sep.node_lists(node_parts, g["num_parts"])
    assert shared.tolist() == g["shared"] and [p.tolist() for p in parts] == g["parts"]


@pytest.mark.parametrize("name,events,num_parts,k,lam", [("c1_tiny", 10000, 4, 0.05, 1.0), ("c1_tiny", 10000, 8, 0.0, 0.3),
                                                         ("c1_tiny", 10000, 3, 0.2, 2.5),
                                                         ("c2_bipartite_medium", 30000, 4, 0.01, 1.0),
                                                         ("c3_bipartite_dense", 30000, 64, 0.05, 1.0)])
def test_assign_matches_oracle(sep, name, events, num_parts, k, lam):
    w = S.WORKLOADS[name].scaled(num_events=events)
    g = S.make_graph(w)
    cent = P.centrality(g.src, g.dst, g.ts, g.num_nodes, beta=1e-5)
    hubs = P.top_k_hubs(cent, k)
    ref_part, A, sizes, _ = P.assign_stream(g.src, g.dst, g.num_nodes, cent, hubs, num_parts, lam, 1e-3)
    is_hub = np.zeros(g.num_nodes, dtype=np.uint8)
    is_hub[hubs] = 1
    part, node_parts, part_edges = sep.assign(sep.make_config(num_parts, 1e-5, k, lam, 1e-3), g.src, g.dst,
                                              g.num_nodes, cent, is_hub)
    assert np.array_equal(part, ref_part)
    assert np.array_equal(node_parts, masks(A))
    assert part_edges.tolist() == sizes
    parts, shared = sep.node_lists(node_parts, num_parts)
    ref_parts, ref_shared = P.node_lists(A, num_parts)
    assert shared.tolist() == ref_shared and [p.tolist() for p in parts] == ref_parts


def test_assign_rejects_bad_arguments(sep):
    from paper_2308_14129_amd import tig
    ok = dict(src=[0, 1], dst=[1, 2], num_nodes=3, cent=[1.0, 1.0, 1.0], is_hub=[0, 0, 0])
    for cfg in (sep.make_config(0, 0.1, 0.0), sep.make_config(65, 0.1, 0.0), sep.make_config(2, 0.1, 0.0, lam=0.0),
                sep.make_config(2, 0.1, 0.0, eps=0.0)):
        with pytest.raises(tig.TigError) as ei:
            sep.assign(cfg, **ok)
        assert ei.value.status == tig.TIG_EINVAL
    with pytest.raises(tig.TigError) as ei:
        sep.assign(sep.make_config(2, 0.1, 0.0), [0, 5], [1, 2], 3, [1.0] * 3, [0] * 3)
    assert ei.value.status == tig.TIG_ERANGE


def test_combine_host_call():
    from paper_2308_14129_amd import pac, tig
    from oracle import pac_oracle as E
    order = np.random.default_rng(11).permutation(8)
    assert pac.combine(order, 4) == E.combine(order, 4)
    assert pac.combine(order, 8) == [1 << int(p) for p in order]
    assert pac.combine(order, 1) == [0xFF]
    for bad in (([0, 1, 2], 2), ([0, 0, 1, 2], 2), ([0, 1, 2, 7], 2)):
        with pytest.raises(tig.TigError):
            pac.combine(*bad)
