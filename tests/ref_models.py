"""Independent small models used to pin the oracle (CPU tests only).

None of this is used by the product or by the oracle; each routine reaches its result by a
different route than ``oracle/grem_oracle.c`` (exact rationals and the paper's two-partition
helper functions; dense matrices; size-level closed forms)."""
from __future__ import annotations

from fractions import Fraction

import numpy as np


def dense_adjacency(rowptr, colidx, n):
    """A[v,u] = number of stored entries (v,u)."""
    A = np.zeros((n, n), dtype=np.int64)
    for v in range(n):
        for e in range(int(rowptr[v]), int(rowptr[v + 1])):
            A[v, int(colidx[e])] += 1
    return A


def brute_cut_entries(A, labels):
    """Entries whose endpoints differ in label (Sec. 1: cut edges), from the dense matrix."""
    lab = np.asarray(labels)
    diff = lab[:, None] != lab[None, :]
    return int((A * diff).sum())


def _assign2(c0, c1, sizes, P):
    """Two-partition choice of the paper's helper `assign` (Alg. 2)."""
    if c0 < c1 and sizes[1] < P:
        return 1
    if c1 < c0 and sizes[0] < P:
        return 0
    return 0 if sizes[0] <= sizes[1] else 1       # arg_min, first index on ties


def sequential_bipartition(rowptr, colidx, n, P, passes, seed=None):
    """The two-partition procedure of Alg. 1 / Alg. 2 run one vertex at a time over the CSR
    rows (vertex v's edges are its row), `passes` times in total, with exact rational averages.
    A node that is being re-assigned is first removed from its partition's size.  Seeded
    vertices keep their label on the first pass and only store their counts (first-chunk
    treatment of Alg. 1)."""
    parts = [-1] * n if seed is None else [int(s) for s in seed]
    sizes = [sum(1 for p in parts if p == 0), sum(1 for p in parts if p == 1)]
    est = [[Fraction(0), Fraction(0)] for _ in range(n)]
    for r in range(passes):
        for v in range(n):
            old = parts[v]
            cnt = [Fraction(0), Fraction(0)]
            for e in range(int(rowptr[v]), int(rowptr[v + 1])):
                p = parts[int(colidx[e])]
                if p != -1:
                    cnt[p] += 1
            if r == 0 and old != -1:
                est[v] = cnt
                continue
            if old != -1:
                cnt = [(est[v][0] + cnt[0]) / 2, (est[v][1] + cnt[1]) / 2]
                sizes[old] -= 1
            new = _assign2(cnt[0], cnt[1], sizes, P)
            sizes[new] += 1
            parts[v] = new
            est[v] = cnt
    return parts, sizes, est


def waterfill_sequence(sizes, count):
    """The partitions picked when `count` items are added one at a time, each to the currently
    smallest partition (lowest id on ties) -- computed level by level, not item by item: at
    level l (the current minimum) every partition whose starting size is <= l receives one item,
    in ascending id."""
    sizes = [int(s) for s in sizes]
    out = []
    level = min(sizes)
    while len(out) < count:
        active = [j for j, s in enumerate(sizes) if s <= level]
        out.extend(active)
        level += 1
    return out[:count]


def edgeless_pass0(n, k, P, chunk):
    """Labels after the first pass on a graph without edges, from partition sizes alone: all
    vertices of a chunk want the smallest partition (lowest id); it takes them in id order while
    it has room; the rest are spread by `waterfill_sequence`."""
    sizes = [0] * k
    labels = np.empty(n, dtype=np.int32)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        m = hi - lo
        t = min(range(k), key=lambda j: (sizes[j], j))
        a = min(m, P - sizes[t])
        labels[lo:lo + a] = t
        sizes[t] += a
        rest = waterfill_sequence(sizes, m - a)
        for i, j in enumerate(rest):
            labels[lo + a + i] = j
            sizes[j] += 1
    return labels


def best_permutation_agreement(labels, planted, k):
    """Largest fraction of vertices on which `labels` agrees with `planted` under a renaming of
    the partitions (k small: all permutations)."""
    from itertools import permutations
    conf = np.zeros((k, k), dtype=np.int64)
    np.add.at(conf, (np.asarray(labels), np.asarray(planted)), 1)
    best = 0
    for perm in permutations(range(k)):
        best = max(best, sum(conf[i, perm[i]] for i in range(k)))
    return best / len(labels)


def sequential_edge_stream(src, dst, n, c_size, P, seed_parts, refine=True):
    """Alg. 1 / Alg. 2 over chunks of an edge list, one node at a time (ascending id inside a chunk),
    every node reading the most recent labels and sizes, exact rational averages, `cnt_nbrs` as the
    literal scan of the chunk's edges.  A node being re-assigned is first removed from its
    partition's size.  With refine=False an assigned node is never looked at again.

    Also reports whether any decision depended on something that changed inside its own chunk:
    a neighbour's label, a size that alters `assign`'s answer, or a partition filled up by this
    chunk's arrivals.  When nothing did, processing the chunk's nodes all at once from the state at
    the chunk's start must give the same result."""
    m = len(src)
    parts = [-1] * n
    sizes = [0, 0]
    est = [[Fraction(0), Fraction(0)] for _ in range(n)]
    dependent = False
    for i in range((m + c_size - 1) // c_size):
        c_edges = [(int(src[e]), int(dst[e])) for e in range(i * c_size, min(m, (i + 1) * c_size))]
        c_nodes = sorted({a for a, _ in c_edges} | {b for _, b in c_edges})

        def cnt_nbrs(node, labels):
            cnt = [Fraction(0), Fraction(0)]
            for a, b in c_edges:
                if a == node or b == node:
                    nbr = a if b == node else b
                    if labels[nbr] != -1:
                        cnt[labels[nbr]] += 1
            return cnt

        if i == 0:
            for v in c_nodes:
                parts[v] = int(seed_parts[v])
            sizes = [parts.count(0), parts.count(1)]
            for v in c_nodes:
                est[v] = cnt_nbrs(v, parts)
            continue
        start_parts, start_sizes, arrivals = list(parts), list(sizes), [0, 0]
        for v in c_nodes:
            old = parts[v]
            if old != -1 and not refine:
                continue
            cnt = cnt_nbrs(v, parts)
            if cnt != cnt_nbrs(v, start_parts):
                dependent = True
            if old != -1:
                cnt = [(est[v][0] + cnt[0]) / 2, (est[v][1] + cnt[1]) / 2]
                sizes[old] -= 1
            new = _assign2(cnt[0], cnt[1], sizes, P)
            at_start = [start_sizes[0] - (old == 0), start_sizes[1] - (old == 1)]
            if new != _assign2(cnt[0], cnt[1], at_start, P):
                dependent = True
            if new != old:
                if start_sizes[new] + arrivals[new] >= P:
                    dependent = True
                arrivals[new] += 1
            sizes[new] += 1
            parts[v] = new
            est[v] = cnt
    return parts, sizes, est, dependent


def chunk_incidence(src, dst, n):
    """M[v,u] = number of listed edges joining v and u, a loop counted once on the diagonal."""
    M = np.zeros((n, n), dtype=np.int64)
    for a, b in zip(src, dst):
        M[int(a), int(b)] += 1
        if a != b:
            M[int(b), int(a)] += 1
    return M
