"""CPU oracle of the streaming edge partitioner (SEP).  TEST INFRASTRUCTURE ONLY.

A plain, sequential statement of the paper's Sec. II-B ("Streaming Edge Partitioning
Component") and its Alg. 1: node centrality with exponential time decay (Eq. 1), the top-k hubs,
the greedy edge stream with its five cases and the score C = C_REP + C_BAL (Eq. 2-6), and the
shared-node list.  Imported only by tests and by the benchmark's CPU-baseline leg; shares no
code with the library and never imports it.  float64 arithmetic throughout.

Readings where the paper is silent (also listed in the design notes):
  * hubs: the floor(k * |V|) nodes of greatest centrality; ties broken towards the smaller id;
  * |p| (partition size in C_BAL), maxsize, minsize: edges assigned to p so far, and the current
    maximum / minimum of that over the partitions (the balance term is the one of the greedy
    heuristic the paper builds on, which counts edges);
  * "restrict replication to hubs": when an endpoint is a non-hub that already resides in a
    partition, that partition is the only candidate (Case 1 says so for one hub + one non-hub;
    the same holds in Case 4/5 when the other endpoint is unassigned);
  * the arg-max over partitions takes the lowest partition index among equal scores;
  * theta when both centralities are 0 (cannot happen for nodes of the stream): 1/2;
  * a node that never occurs in the stream belongs to no partition.

Pins (tests/test_sep_oracle.py): a six-node stream assigned by hand, Eq. 1 closed forms, Theorem 1
(RF <= k|P| + (1 - k)), only hubs are ever replicated, edges are discarded in Case 3 only,
k = 0 degenerates to "no shared nodes", every kept edge lies inside one partition's node list.
"""
from __future__ import annotations

import numpy as np


def centrality(src, dst, ts, num_nodes, beta):
    """Eq. 1: Cent(i) = sum over the events incident to i of exp(beta * (t - t_max)),
    accumulated in stream order."""
    cent = np.zeros(num_nodes, dtype=np.float64)
    if len(ts) == 0:
        return cent
    t_max = float(np.max(ts))
    for s, d, t in zip(src, dst, ts):
        w = np.exp(beta * (float(t) - t_max))
        cent[s] += w
        cent[d] += w
    return cent


def top_k_hubs(cent, k_frac):
    """The floor(k * |V|) nodes of greatest centrality (ties: smaller id first), as a sorted id list."""
    n = int(np.floor(k_frac * len(cent)))
    order = sorted(range(len(cent)), key=lambda i: (-cent[i], i))
    return sorted(order[:n])


def assign_stream(src, dst, num_nodes, cent, hubs, num_parts, lam, eps):
    """Alg. 1, the edge loop.  Returns (edge_part [E] with -1 for a discarded edge,
    A: list of sets of partitions per node, sizes: edges per partition, margins: the smallest
    difference between the best and the second-best score met in an arg-max with more than one
    candidate, which tells a test how close any decision was to a tie)."""
    is_hub = np.zeros(num_nodes, dtype=bool)
    is_hub[list(hubs)] = True
    A = [set() for _ in range(num_nodes)]
    sizes = [0] * num_parts
    edge_part = np.full(len(src), -1, dtype=np.int32)
    margin = np.inf

    def theta(i, j):
        tot = cent[i] + cent[j]
        return 0.5 if tot == 0.0 else cent[i] / tot

    def h(i, j, p):  # Eq. 5
        return 1.0 + (1.0 - theta(i, j)) if p in A[i] else 0.0

    def best(i, j, cands):
        nonlocal margin
        mx, mn = max(sizes), min(sizes)
        scores = []
        for p in cands:
            c_rep = h(i, j, p) + h(j, i, p)                      # Eq. 4
            c_bal = lam * (mx - sizes[p]) / (eps + mx - mn)      # Eq. 6
            scores.append(c_rep + c_bal)                         # Eq. 3
        top = max(scores)
        if len(scores) > 1:
            rest = sorted(scores)[-2]
            if top - rest > 0.0:
                margin = min(margin, top - rest)
        return cands[scores.index(top)]

    everything = list(range(num_parts))
    for e, (i, j) in enumerate(zip(src, dst)):
        i, j = int(i), int(j)
        ai, aj = bool(A[i]), bool(A[j])
        if ai and aj:
            if is_hub[i] != is_hub[j]:                           # Case 1
                low = j if is_hub[i] else i
                p = next(iter(A[low]))
            elif is_hub[i] and is_hub[j]:                        # Case 2
                p = best(i, j, everything)
            else:                                                # Case 3
                p = next(iter(A[i])) if A[i] == A[j] else -1
        else:                                                    # Case 4 & 5
            fixed = [n for n in (i, j) if A[n] and not is_hub[n]]
            p = next(iter(A[fixed[0]])) if fixed else best(i, j, everything)
        if p >= 0:
            edge_part[e] = p
            A[i].add(p)
            A[j].add(p)
            sizes[p] += 1
    return edge_part, A, sizes, margin


def node_lists(A, num_parts):
    """Alg. 1, the node loop: nodes with replicas in more than one partition go to the shared
    list and to every partition; every other assigned node to its one partition."""
    shared = [i for i, a in enumerate(A) if len(a) > 1]
    parts = [[] for _ in range(num_parts)]
    for i, a in enumerate(A):
        if len(a) > 1:
            for p in range(num_parts):
                parts[p].append(i)
        elif len(a) == 1:
            parts[next(iter(a))].append(i)
    return parts, shared


def partition(src, dst, ts, num_nodes, num_parts, beta, k_frac, lam, eps):
    cent = centrality(src, dst, ts, num_nodes, beta)
    hubs = top_k_hubs(cent, k_frac)
    edge_part, A, sizes, margin = assign_stream(src, dst, num_nodes, cent, hubs, num_parts, lam, eps)
    parts, shared = node_lists(A, num_parts)
    return {"cent": cent, "hubs": hubs, "edge_part": edge_part, "A": A, "sizes": sizes,
            "parts": parts, "shared": shared, "margin": margin}


def replication_factor(parts, num_nodes_present):
    """RF = total node replicas / total number of nodes (nodes that occur in the stream)."""
    return sum(len(p) for p in parts) / max(1, num_nodes_present)


def edge_cut(edge_part):
    """EC = discarded edges / edges."""
    return float(np.mean(edge_part < 0)) if len(edge_part) else 0.0
