"""Offline construction of the index bijection `f_index` (paper Section III-G, "Index Bijection via
Local-Global Information Fusion", and the index-graph algorithm of that section).

The hot path takes the result as the optional `remap` argument of `tt_index_reorder`: rows that are
looked up together get neighbouring new indices, so that they share TT prefixes `(i1, i2)` and the
prefix products and partial gradients are reused more often.  This module is host-side
preprocessing (numpy), done once before training as the paper says; nothing here runs per batch.

Steps, in the paper's order:
  1. global information: rows ranked by access frequency over the sample batches; the first
     `hot_ratio * num_rows` ranks are the hot rows, which keep their frequency order and are not
     part of the graph;
  2. local information: an index graph over the remaining rows that occur in the sample, with an
     edge (weight = number of co-occurrences) between two rows looked up in the same group.  The
     paper pairs all rows of a mini-batch; `group="bag"` (default) pairs the rows of one bag, which
     is what carries signal for multi-hot features, and `group="batch"` follows the paper literally.
     A group with more than `max_group` distinct nodes keeps its `max_group` smallest ones (the most
     frequent rows), the pair count being quadratic.  With `device="cuda"` the edges of a batch are
     generated on the GPU by the library's `tt_index_graph_edges` job (pair generation per bag, two
     stable radix sorts, run heads) with the same rule, and merged across batches here;
  3. communities by greedy modularity maximisation (local moving of single nodes, the first phase
     of the Louvain method, in a seeded order until no move improves the modularity
     Q = sum_c [ e_cc / 2m - (k_c / 2m)^2 ]);
  4. new indices: hot rows first (by rank), then the communities one after the other (largest
     total frequency first, members by rank), then the rows never seen, in their old order.

Readings of the paper (it gives no code for steps 3-4): the modularity formula is printed without
the inner normalisation and is read as the standard one above; "assigned sequentially" is read as
step 4.  There is no reference result to compare with: the construction is judged by the reuse it
produces (`prefix_reuse_stats`), and `tests/test_bijection.py` checks that it is a bijection, is
deterministic, and recovers planted communities.
"""
from __future__ import annotations

import numpy as np


def frequency_order(batches, num_rows: int):
    """rank[row] = position of the row when rows are sorted by decreasing access count (ties by
    row id); rows never accessed come last in their old order.  Returns (rank, counts)."""
    counts = np.zeros(num_rows, dtype=np.int64)
    for idx in batches:
        idx = np.asarray(idx)
        idx = idx[(idx >= 0) & (idx < num_rows)]
        counts += np.bincount(idx, minlength=num_rows)
    order = np.lexsort((np.arange(num_rows), -counts))  # by count descending, then by row id
    rank = np.empty(num_rows, dtype=np.int64)
    rank[order] = np.arange(num_rows)
    return rank, counts


def _merge_edges(us, vs, ws):
    if not us:
        return np.zeros(0, np.int64), np.zeros(0, np.int64), np.zeros(0, np.int64)
    u, v, w = np.concatenate(us), np.concatenate(vs), np.concatenate(ws)
    base = int(v.max()) + 1
    uniq, inv = np.unique(u * base + v, return_inverse=True)
    return uniq // base, uniq % base, np.bincount(inv, weights=w, minlength=uniq.size).astype(np.int64)


def index_graph_edges(batches, rank, hot_thresh: int, group: str = "bag", max_group: int = 64, bag_cap: int = 256):
    """Weighted edge list (u, v, w), u < v, sorted by (u, v), over frequency ranks shifted by the hot
    threshold (the paper's clamp-and-subtract: every hot row collapses to node 0, which is dropped)."""
    us, vs = [], []
    for item in batches:
        if group == "bag":
            idx, off = item
            groups = [np.asarray(idx[off[b]:off[b + 1]])[:bag_cap] for b in range(len(off) - 1)]
        else:
            groups = [np.asarray(item[0] if isinstance(item, tuple) else item)]
        for grp in groups:
            grp = grp[(grp >= 0) & (grp < rank.size)]
            node = np.unique(np.maximum(rank[grp], hot_thresh) - hot_thresh)
            node = node[node > 0][:max_group]  # node 0 = the hot rows; the smallest max_group nodes are kept
            if node.size < 2:
                continue
            a, b = np.triu_indices(node.size, k=1)
            us.append(node[a])
            vs.append(node[b])
    return _merge_edges(us, vs, [np.ones(len(x), np.int64) for x in us])


def index_graph_edges_gpu(batches, rank, hot_thresh: int, max_group: int = 64):
    """The same edge list with the per-batch work done by the GPU job (bags as groups)."""
    import torch

    from . import binding
    d_rank = torch.from_numpy(np.ascontiguousarray(rank, dtype=np.int32)).cuda()
    us, vs, ws = [], [], []
    for idx, off in batches:
        d_idx = torch.from_numpy(np.ascontiguousarray(idx, dtype=np.int64)).cuda()
        d_off = torch.from_numpy(np.ascontiguousarray(off, dtype=np.int64)).cuda()
        u, v, w = binding.tt_index_graph_edges(d_idx, d_off, d_rank, hot_thresh, max_group)
        us.append(u.cpu().numpy().astype(np.int64))
        vs.append(v.cpu().numpy().astype(np.int64))
        ws.append(w.cpu().numpy().astype(np.int64))
    return _merge_edges(us, vs, ws)


def greedy_modularity_communities(u, v, w, max_sweeps: int = 20, seed: int = 0):
    """Community label per node id occurring in the edge list (dict node -> label): nodes are moved
    one at a time to the neighbouring community with the largest modularity gain until a sweep
    moves nothing."""
    nodes = np.unique(np.concatenate([u, v])) if len(u) else np.zeros(0, np.int64)
    if nodes.size == 0:
        return {}
    pos = {int(n): i for i, n in enumerate(nodes)}
    n = nodes.size
    nbr = [dict() for _ in range(n)]
    for a, b, c in zip(u.tolist(), v.tolist(), w.tolist()):
        ia, ib = pos[a], pos[b]
        nbr[ia][ib] = nbr[ia].get(ib, 0) + c
        nbr[ib][ia] = nbr[ib].get(ia, 0) + c
    deg = np.array([sum(d.values()) for d in nbr], dtype=np.float64)
    two_m = float(deg.sum())
    label = np.arange(n)
    tot = deg.copy()  # total degree per community
    order = np.random.default_rng(seed).permutation(n)
    for _ in range(max_sweeps):
        moved = 0
        for i in order.tolist():
            li = int(label[i])
            links = {}
            for j, c in nbr[i].items():
                lj = int(label[j])
                links[lj] = links.get(lj, 0.0) + c
            tot[li] -= deg[i]
            best, best_gain = li, links.get(li, 0.0) - tot[li] * deg[i] / two_m
            for lj in sorted(links):  # sorted: ties resolve the same way in every run
                gain = links[lj] - tot[lj] * deg[i] / two_m
                if gain > best_gain + 1e-12:
                    best, best_gain = lj, gain
            tot[best] += deg[i]
            if best != li:
                label[i] = best
                moved += 1
        if moved == 0:
            break
    return {int(nodes[i]): int(label[i]) for i in range(n)}


def build_index_bijection(batches, num_rows: int, hot_ratio: float = 0.001, group: str = "bag",
                          max_group: int = 64, seed: int = 0, device: str = "cpu"):
    """remap[old row] = new row, an int64 permutation of range(num_rows), from sample `batches`
    (a list of (indices, offsets) pairs, CSR offsets of length bags + 1)."""
    flat = [np.asarray(b[0]) for b in batches]
    rank, counts = frequency_order(flat, num_rows)
    hot_thresh = int(num_rows * hot_ratio)
    if device == "cuda":
        if group != "bag":
            raise ValueError("the GPU edge job pairs the rows of one bag")
        u, v, w = index_graph_edges_gpu(batches, rank, hot_thresh, max_group=max_group)
    else:
        u, v, w = index_graph_edges(batches, rank, hot_thresh, group=group, max_group=max_group)
    comm = greedy_modularity_communities(u, v, w, seed=seed)
    by_rank = np.argsort(rank, kind="stable")  # row with rank r
    new_of_rank = np.full(num_rows, -1, dtype=np.int64)
    nxt = 0
    for r in range(min(hot_thresh, num_rows)):  # hot rows keep their frequency order
        new_of_rank[r] = nxt
        nxt += 1
    groups = {}
    for node, lab in comm.items():
        groups.setdefault(lab, []).append(node + hot_thresh)  # back to ranks
    weight = {lab: -int(sum(counts[by_rank[r]] for r in members)) for lab, members in groups.items()}
    for lab in sorted(groups, key=lambda x: (weight[x], min(groups[x]))):
        for r in sorted(groups[lab]):
            new_of_rank[r] = nxt
            nxt += 1
    rest = np.flatnonzero(new_of_rank < 0)  # seen but isolated rows by rank, then the never-seen rows
    new_of_rank[rest] = np.arange(nxt, nxt + rest.size)
    remap = np.empty(num_rows, dtype=np.int64)
    remap[by_rank] = new_of_rank
    return remap


def prefix_reuse_stats(batches, n, remap=None):
    """Mean number of distinct rows and of distinct TT prefixes (i1, i2) per batch: the quantity the
    bijection is meant to lower (every distinct prefix costs one prefix product forward and three
    backward)."""
    rows, prefs = [], []
    for item in batches:
        idx = np.asarray(item[0] if isinstance(item, tuple) else item)
        if remap is not None:
            idx = remap[idx]
        rows.append(np.unique(idx).size)
        prefs.append(np.unique(idx // n[2]).size)
    return float(np.mean(rows)), float(np.mean(prefs))
