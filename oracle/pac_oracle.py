"""CPU oracle of the epoch machinery of parallel training on partitions.  TEST INFRASTRUCTURE ONLY.

Plain statements of the paper's Sec. II-C "Distributed Parallel Training" and its Alg. 2, as one
machine sees them when it holds several partitions at once:
  * sub-graph of a partition: E_k = {(i, j, t) in E | i, j in V_k}, with the shared nodes of the
    partitioner (more than one replica) members of every V_k;
  * shuffle-and-combine: the |P| small parts are shuffled and joined, in order, into N groups;
    a group's node set is the union of its parts' node sets, so its sub-graph regains the edges
    that ran between its parts;
  * the training loop of Alg. 2: every partition cycles over its own batches, resets its memory
    at the start of a data cycle and backs it up at the end of one, until the partition with the
    most batches has finished one cycle; then every memory is restored from its latest backup;
  * memory synchronisation of the shared nodes: every replica takes the row with the largest
    last-update time across the partitions (ties: the lowest partition), or the mean of the rows.
Imported only by tests; shares no code with the library and never imports it.

Readings where the paper is silent: the parts of a group are consecutive entries of the shuffled
order (|P| / N each); the loop stops after max_k(number of batches of k) steps, the first moment
"all GPUs have finished at least one complete traversal"; local node ids of a sub-graph are the
ranks of its members in id order; the mean rule keeps the largest last-update time.
"""
from __future__ import annotations

import numpy as np

from . import tig_oracle as O


def effective_masks(node_parts, num_parts):
    """Alg. 1's node loop: a node with replicas in more than one part resides in every part."""
    node_parts = np.asarray(node_parts, dtype=np.uint64)
    bits = np.array([bin(int(m)).count("1") for m in node_parts])
    full = np.uint64((1 << num_parts) - 1)
    return np.where(bits > 1, full, node_parts)


def combine(order, num_groups):
    """Group masks of the shuffled parts: group g joins entries g*w .. g*w + w - 1 of `order`."""
    w = len(order) // num_groups
    assert w * num_groups == len(order)
    return [sum(1 << int(p) for p in order[g * w:(g + 1) * w]) for g in range(num_groups)]


def members(node_parts, num_parts, group_mask):
    eff = effective_masks(node_parts, num_parts)
    return (eff & np.uint64(group_mask)) != 0


def subgraph(src, dst, node_parts, num_parts, group_mask):
    """Event ids of E_k (chronological), local id of every node (-1: not a member), member count."""
    m = members(node_parts, num_parts, group_mask)
    eids = np.flatnonzero(m[src] & m[dst])
    local = np.full(len(m), -1, dtype=np.int32)
    local[m] = np.arange(int(m.sum()), dtype=np.int32)
    return eids, local, int(m.sum())


def epoch(parts, K, H, deferred=False):
    """Alg. 2 on several partitions in lock step.  parts: dicts with num_nodes, mem_dim, src, dst, ts,
    edge_feat, W, batch, neg (one negative per event or None).  Returns the final states and, per
    partition, the list of (global step, batch index, reset?, backup?) it went through."""
    states = [O.OracleState.zeros(p["num_nodes"], p["mem_dim"]) for p in parts]
    backups = [None] * len(parts)
    n_batches = [(len(p["src"]) + p["batch"] - 1) // p["batch"] for p in parts]
    trace = [[] for _ in parts]
    step = 0
    done = [False] * len(parts)
    while True:
        for k, p in enumerate(parts):
            i = step % n_batches[k]
            loop_start, loop_end = i == 0, i == n_batches[k] - 1
            if loop_start:
                states[k] = O.OracleState.zeros(p["num_nodes"], p["mem_dim"])
            first = i * p["batch"]
            count = min(p["batch"], len(p["src"]) - first)
            neg = None if p.get("neg") is None else p["neg"][first:first + count]
            O.step(states[k], p["src"], p["dst"], p["ts"], p["edge_feat"], p["W"], first, count, neg, K, H,
                   deferred=deferred)
            if loop_end:
                backups[k] = states[k].copy()
                done[k] = True
            trace[k].append((step, i, loop_start, loop_end))
        step += 1
        if all(done):
            break
    final = [b.copy() for b in backups]
    for st in final:
        st.drop_pending()  # a restored memory carries no messages kept for a next step
    return final, trace, step


def sync_shared(states, local_ids, mode="latest"):
    """states: OracleState per partition; local_ids[k][s]: row of shared node s in partition k."""
    n = len(states)
    for s in range(len(local_ids[0])):
        rows = [int(local_ids[k][s]) for k in range(n)]
        times = [states[k].last_update[rows[k]] for k in range(n)]
        t_star = max(times)
        if mode == "latest":
            win = times.index(t_star)
            row = states[win].mem[rows[win]].copy()
        else:
            acc = states[0].mem[rows[0]].astype(np.float32).copy()
            for k in range(1, n):
                acc = (acc + states[k].mem[rows[k]]).astype(np.float32)
            row = (acc / np.float32(n)).astype(np.float32)
        for k in range(n):
            states[k].mem[rows[k]] = row
            states[k].last_update[rows[k]] = t_star
