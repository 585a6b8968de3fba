"""Seeded synthetic graphs shaped like the paper's partitioning workloads (Sec. 6, "Datasets,
Models, and Metrics": OGBN-Papers100M has 111M nodes and 1.6B edges; the partitioner's input is
an edge list in random order, Sec. 4.1).

This module only builds inputs: undirected graphs as symmetrised CSR (rows sorted by column id,
self-loops removed, duplicates removed, int32 column ids, vertex ids randomly permuted so that the
stream order is random).  It contains none of the partitioner's arithmetic and imports neither the
GPU binding nor the CPU oracle; both are fed from here.

Small graphs come back as numpy arrays; the large generators run with torch on whatever device is
asked for (a GPU for the full-size workloads) and return torch tensors on that device.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch


@dataclass
class Graph:
    rowptr: object   # (n+1,) int32 or int64; numpy array or torch tensor
    colidx: object   # (nnz,) int32
    n: int
    nnz: int
    directed_edges: int            # number of directed samples / input edges before symmetrising
    planted: Optional[object] = None   # planted block per vertex, when the model has one
    name: str = ""


# --------------------------------------------------------------------------------------------
# numpy side: tiny graphs and the planted-partition model
# --------------------------------------------------------------------------------------------

def csr_from_pairs_np(u: np.ndarray, v: np.ndarray, n: int, rowptr_dtype=np.int64,
                      symmetrise: bool = True, dedup: bool = True, drop_loops: bool = True):
    """CSR of the listed pairs; by default both directions, no loops, no duplicates."""
    u = np.asarray(u, dtype=np.int64)
    v = np.asarray(v, dtype=np.int64)
    if symmetrise:
        r = np.concatenate([u, v])
        c = np.concatenate([v, u])
    else:
        r, c = u, v
    if drop_loops:
        keep = r != c
        r, c = r[keep], c[keep]
    key = r * n + c
    key = np.unique(key) if dedup else np.sort(key, kind="stable")
    r = key // n
    c = (key % n).astype(np.int32)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(r, minlength=n), out=rowptr[1:])
    return rowptr.astype(rowptr_dtype), c


def _sample_pairs_without_replacement(rng, npairs: int, count: int) -> np.ndarray:
    """`count` distinct integers of [0, npairs), uniformly."""
    if count == 0:
        return np.empty(0, dtype=np.int64)
    got = np.unique(rng.integers(0, npairs, size=count, dtype=np.int64))
    while got.size < count:
        more = rng.integers(0, npairs, size=(count - got.size) * 2 + 8, dtype=np.int64)
        got = np.unique(np.concatenate([got, more]))
        if got.size > count:
            got = rng.permutation(got)[:count]
            got.sort()
    return got


def planted_partition(n: int = 10_000, blocks: int = 4, mean_degree: float = 10.0,
                      ratio: float = 20.0, seed: int = 0, rowptr_dtype=np.int32) -> Graph:
    """Planted-partition (stochastic block) model: `blocks` equal blocks; every unordered pair is
    an edge independently with probability p_in (same block) or p_out, p_in = ratio * p_out,
    scaled so that the expected degree is `mean_degree`.  Vertex ids are randomly permuted."""
    assert n % blocks == 0
    rng = np.random.default_rng(seed)
    b = n // blocks
    p_out = mean_degree / (ratio * (b - 1) + (n - b))
    p_in = ratio * p_out
    us, vs = [], []
    for i in range(blocks):
        for j in range(i, blocks):
            if i == j:
                npairs = b * (b - 1) // 2
                m = rng.binomial(npairs, p_in)
                idx = _sample_pairs_without_replacement(rng, npairs, m)
                # unrank idx -> (a, c) with a < c in [0, b)
                a = np.floor((1 + np.sqrt(1 + 8 * idx.astype(np.float64))) / 2).astype(np.int64)
                a = np.where(a * (a - 1) // 2 > idx, a - 1, a)
                a = np.where((a + 1) * a // 2 <= idx, a + 1, a)
                c = idx - a * (a - 1) // 2
                us.append(i * b + a)
                vs.append(i * b + c)
            else:
                npairs = b * b
                m = rng.binomial(npairs, p_out)
                idx = _sample_pairs_without_replacement(rng, npairs, m)
                us.append(i * b + idx // b)
                vs.append(j * b + idx % b)
    u = np.concatenate(us)
    v = np.concatenate(vs)
    perm = rng.permutation(n)            # new id of old vertex i
    planted_old = np.repeat(np.arange(blocks, dtype=np.int32), b)
    planted = np.empty(n, dtype=np.int32)
    planted[perm] = planted_old
    rowptr, colidx = csr_from_pairs_np(perm[u], perm[v], n, rowptr_dtype=rowptr_dtype)
    return Graph(rowptr, colidx, n, int(colidx.size), int(u.size), planted,
                 f"planted-partition n={n} blocks={blocks} deg={mean_degree} ratio={ratio} seed={seed}")


def random_graph_np(n: int, m: int, seed: int, rowptr_dtype=np.int64, simple: bool = True) -> Graph:
    """`m` uniformly random pairs; `simple=False` keeps loops and duplicates and does not
    symmetrise (for tests of how stored entries are counted)."""
    rng = np.random.default_rng(seed)
    u = rng.integers(0, n, size=m)
    v = rng.integers(0, n, size=m)
    if simple:
        rowptr, colidx = csr_from_pairs_np(u, v, n, rowptr_dtype)
    else:
        rowptr, colidx = csr_from_pairs_np(u, v, n, rowptr_dtype, symmetrise=False, dedup=False,
                                           drop_loops=False)
    return Graph(rowptr, colidx, n, int(colidx.size), m, None, f"uniform n={n} m={m} seed={seed}")


# --------------------------------------------------------------------------------------------
# torch side: R-MAT, Chung-Lu, hub stress (any device; sized for > 2^31 entries)
# --------------------------------------------------------------------------------------------

_BLOCK_ENTRIES = 1 << 27   # target entries per sorted block (torch.sort takes < 2^31 elements)
_SEGMENT = 1 << 30         # samples per boolean-mask / index operation


def csr_from_samples(src: torch.Tensor, dst: torch.Tensor, n: int, rowptr_dtype=torch.int64,
                     block_entries: int = _BLOCK_ENTRIES):
    """Symmetrised, loop-free, deduplicated CSR of the directed samples (src[i], dst[i]).
    Works row-range by row-range so that no single sort exceeds `block_entries` by much."""
    dev = src.device
    M = src.numel()
    nblocks = max(1, math.ceil(2 * M / block_entries))
    rows_per_block = math.ceil(n / nblocks)
    deg = torch.zeros(n, dtype=torch.int64, device=dev)
    pieces = []
    for b in range(nblocks):
        lo = b * rows_per_block
        hi = min(n, lo + rows_per_block)
        if lo >= hi:
            break
        # masks over at most _SEGMENT samples at a time (boolean indexing of longer tensors overflows)
        rparts, cparts = [], []
        for s0 in range(0, M, _SEGMENT):
            ss, dd = src[s0:s0 + _SEGMENT], dst[s0:s0 + _SEGMENT]
            m1 = (ss >= lo) & (ss < hi)
            m2 = (dd >= lo) & (dd < hi)
            rparts += [ss[m1], dd[m2]]
            cparts += [dd[m1], ss[m2]]
            del m1, m2
        rows = torch.cat(rparts).to(torch.int64)
        cols = torch.cat(cparts).to(torch.int64)
        del rparts, cparts
        keep = rows != cols
        key = ((rows[keep] - lo) << 32) | cols[keep]
        del rows, cols, keep
        key = torch.sort(key).values
        key = torch.unique_consecutive(key)
        pieces.append((key & 0xFFFFFFFF).to(torch.int32))
        r = key >> 32
        deg[lo:hi] = torch.bincount(r, minlength=hi - lo)
        del key, r
    colidx = torch.cat(pieces) if len(pieces) > 1 else pieces[0]
    del pieces
    rowptr = torch.zeros(n + 1, dtype=torch.int64, device=dev)
    torch.cumsum(deg, 0, out=rowptr[1:])
    return rowptr.to(rowptr_dtype), colidx


def _rmat_samples(scale: int, m: int, abcd, gen: torch.Generator, device, batch: int = 1 << 27):
    a, b, c, _ = abcd
    src = torch.empty(m, dtype=torch.int32, device=device)
    dst = torch.empty(m, dtype=torch.int32, device=device)
    for s in range(0, m, batch):
        e = min(m, s + batch)
        si = torch.zeros(e - s, dtype=torch.int32, device=device)
        di = torch.zeros(e - s, dtype=torch.int32, device=device)
        for _level in range(scale):
            u = torch.rand(e - s, generator=gen, device=device)
            sbit = (u >= a + b).to(torch.int32)
            dbit = (((u >= a) & (u < a + b)) | (u >= a + b + c)).to(torch.int32)
            si = (si << 1) | sbit
            di = (di << 1) | dbit
        src[s:e] = si
        dst[s:e] = di
    return src, dst


def _permutation(n: int, gen: torch.Generator, device) -> torch.Tensor:
    return torch.randperm(n, generator=gen, device=device).to(torch.int32)


def rmat(scale: int, edge_factor: int = 16, abcd=(0.57, 0.19, 0.19, 0.05), seed: int = 0,
         device="cpu", rowptr_dtype=torch.int32) -> Graph:
    """R-MAT: edge_factor * 2^scale directed samples, one quadrant choice per bit level, no
    noise; ids permuted; loops dropped; symmetrised; deduplicated."""
    n = 1 << scale
    m = edge_factor * n
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    src, dst = _rmat_samples(scale, m, abcd, gen, device)
    perm = _permutation(n, gen, device)
    for s0 in range(0, m, _SEGMENT):
        src[s0:s0 + _SEGMENT] = perm[src[s0:s0 + _SEGMENT].long()]
        dst[s0:s0 + _SEGMENT] = perm[dst[s0:s0 + _SEGMENT].long()]
    rowptr, colidx = csr_from_samples(src, dst, n, rowptr_dtype)
    return Graph(rowptr, colidx, n, int(colidx.numel()), m, None,
                 f"rmat scale={scale} ef={edge_factor} seed={seed}")


def _chung_lu_offset(n: int, m: int, alpha: float, cap: float) -> float:
    """Offset i0 of the rank weights w_i ~ integral of x^-alpha over [i+i0, i+i0+1) such that the
    heaviest vertex has expected symmetrised degree `cap` (2*m endpoint draws in total)."""
    q = 1.0 - alpha

    def top_degree(i0):
        tot = (n + i0) ** q - i0 ** q
        return 2.0 * m * ((i0 + 1.0) ** q - i0 ** q) / tot

    lo, hi = 1e-9, float(n)
    if top_degree(lo) <= cap:
        return lo
    for _ in range(200):
        mid = math.sqrt(lo * hi)
        if top_degree(mid) > cap:
            lo = mid
        else:
            hi = mid
    return hi


def chung_lu(n: int, m: int, gamma: float = 2.1, cap: float = 50_000.0, seed: int = 0, device="cpu",
             rowptr_dtype=torch.int64, batch: int = 1 << 27) -> Graph:
    """Chung-Lu power-law graph by endpoint sampling: `m` directed samples whose two endpoints are
    drawn independently with probability proportional to w_i, w_i the mass of x^(-1/(gamma-1)) on
    [i+i0, i+i0+1); i0 is set so that the largest expected degree equals `cap`.  Ids permuted,
    loops dropped, symmetrised, deduplicated."""
    alpha = 1.0 / (gamma - 1.0)
    q = 1.0 - alpha
    i0 = _chung_lu_offset(n, m, alpha, cap)
    lo_q = i0 ** q
    span_q = (n + i0) ** q - lo_q
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    perm = _permutation(n, gen, device)

    def draw(count):
        u = torch.rand(count, generator=gen, device=device, dtype=torch.float64)
        x = (lo_q + u * span_q).pow_(1.0 / q)
        r = (x - i0).floor_().clamp_(0, n - 1).to(torch.int64)
        return perm[r]

    src = torch.empty(m, dtype=torch.int32, device=device)
    dst = torch.empty(m, dtype=torch.int32, device=device)
    for s in range(0, m, batch):
        e = min(m, s + batch)
        src[s:e] = draw(e - s)
        dst[s:e] = draw(e - s)
    rowptr, colidx = csr_from_samples(src, dst, n, rowptr_dtype)
    return Graph(rowptr, colidx, n, int(colidx.numel()), m, None,
                 f"chung-lu n={n} m={m} gamma={gamma} cap={cap} seed={seed}")


def hub_stress(scale: int = 24, edge_factor: int = 16, hubs: int = 64, hub_degree: int = 2_000_000,
               abcd=(0.57, 0.19, 0.19, 0.05), seed: int = 0, device="cpu",
               rowptr_dtype=torch.int32) -> Graph:
    """R-MAT as `rmat`, plus `hubs` distinct vertices each joined to `hub_degree` distinct
    uniformly chosen other vertices."""
    n = 1 << scale
    if hub_degree >= n or hubs > n:
        raise ValueError("hub_stress: a hub has at most n - 1 distinct neighbours, and there are at most n hubs")
    m = edge_factor * n
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    src, dst = _rmat_samples(scale, m, abcd, gen, device)
    perm = _permutation(n, gen, device)
    src = perm[src.long()]
    dst = perm[dst.long()]
    hub_ids = torch.randperm(n, generator=gen, device=device)[:hubs].to(torch.int32)
    hs, hd = [src], [dst]
    for i in range(hubs):
        tgt = torch.randperm(n, generator=gen, device=device)[:hub_degree].to(torch.int32)
        hs.append(hub_ids[i].expand(hub_degree).contiguous())
        hd.append(tgt)
    src = torch.cat(hs)
    dst = torch.cat(hd)
    del hs, hd
    rowptr, colidx = csr_from_samples(src, dst, n, rowptr_dtype)
    return Graph(rowptr, colidx, n, int(colidx.numel()), m + hubs * hub_degree, None,
                 f"hub-stress scale={scale} ef={edge_factor} hubs={hubs}x{hub_degree} seed={seed}")


def to_numpy(g: Graph) -> Graph:
    """Host numpy copy of a torch-backed graph."""
    if isinstance(g.rowptr, np.ndarray):
        return g
    return Graph(g.rowptr.cpu().numpy(), g.colidx.cpu().numpy(), g.n, g.nnz, g.directed_edges,
                 None if g.planted is None else g.planted.cpu().numpy(), g.name)


# --------------------------------------------------------------------------------------------
# edge lists in random order (the partitioner's input as the paper states it, Sec. 4.1)
# --------------------------------------------------------------------------------------------

@dataclass
class EdgeStream:
    src: object      # (m,) int32; numpy array or torch tensor
    dst: object      # (m,) int32
    n: int
    m: int
    name: str = ""


def edge_stream(g: Graph, seed: int = 0) -> EdgeStream:
    """Every undirected edge of a symmetric CSR once, in random order and with a random orientation.
    Works on numpy- and torch-backed graphs (the result lives where the graph does)."""
    if isinstance(g.rowptr, np.ndarray):
        rng = np.random.default_rng(seed)
        deg = np.diff(g.rowptr.astype(np.int64))
        rows = np.repeat(np.arange(g.n, dtype=np.int64), deg)
        cols = g.colidx.astype(np.int64)
        keep = rows <= cols
        s, d = rows[keep], cols[keep]
        order = rng.permutation(s.size)
        s, d = s[order], d[order]
        flip = rng.random(s.size) < 0.5
        s, d = np.where(flip, d, s), np.where(flip, s, d)
        return EdgeStream(s.astype(np.int32), d.astype(np.int32), g.n, int(s.size),
                          f"edge stream of [{g.name}] seed={seed}")
    dev = g.colidx.device
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    # upper-triangle entries, one segment of rows at a time so that no temporary exceeds a few GB
    parts_s, parts_d = [], []
    rowptr = g.rowptr.to(torch.int64)
    lo = 0
    while lo < g.n:
        # rows whose entries fill about one segment
        target = int(rowptr[lo].item()) + _SEGMENT // 4
        hi = int(torch.searchsorted(rowptr, torch.tensor([target], device=dev)).item())
        hi = min(max(hi, lo + 1), g.n)
        a, b = int(rowptr[lo].item()), int(rowptr[hi].item())
        deg = (rowptr[lo + 1:hi + 1] - rowptr[lo:hi])
        rows = torch.repeat_interleave(torch.arange(lo, hi, device=dev, dtype=torch.int32), deg)
        cols = g.colidx[a:b]
        keep = rows <= cols
        parts_s.append(rows[keep])
        parts_d.append(cols[keep])
        del rows, cols, keep, deg
        lo = hi
    s = torch.cat(parts_s)
    d = torch.cat(parts_d)
    del parts_s, parts_d
    s, d = _shuffle_pairs(s, d, gen)
    m = int(s.numel())
    for a in range(0, m, _SEGMENT):          # random orientation, a segment at a time
        b = min(m, a + _SEGMENT)
        flip = torch.rand(b - a, generator=gen, device=dev) < 0.5
        sa, da = s[a:b].clone(), d[a:b]
        s[a:b] = torch.where(flip, da, sa)
        d[a:b] = torch.where(flip, sa, da)
        del flip, sa, da
    return EdgeStream(s, d, g.n, m, f"edge stream of [{g.name}] seed={seed}")


def _shuffle_pairs(s: torch.Tensor, d: torch.Tensor, gen: torch.Generator):
    """Both arrays in one uniformly random order.  Up to 2^30 elements this is one random permutation;
    longer arrays are cut in two halves, each half is permuted, and the halves are merged by a random
    pattern holding exactly as many positions for each half as it has elements (a random permutation
    restricted to two blocks is exactly that)."""
    m, dev = int(s.numel()), s.device
    if m <= _SEGMENT:
        order = _permutation(m, gen, dev)
        return s[order], d[order]
    if m > 2 * _SEGMENT:
        raise ValueError("edge lists longer than 2^31 are not generated")
    h = m // 2
    pattern = torch.empty(m, dtype=torch.bool, device=dev)      # True: the position takes from the first half
    for a in range(0, m, _SEGMENT):
        b = min(m, a + _SEGMENT)
        pattern[a:b] = torch.rand(b - a, generator=gen, device=dev) < (h / m)
    # make the count exact by flipping randomly chosen positions of the surplus kind in the first segment
    surplus = sum(int(pattern[a:min(m, a + _SEGMENT)].sum().item()) for a in range(0, m, _SEGMENT)) - h
    if surplus != 0:
        head = pattern[:_SEGMENT]
        where = torch.nonzero(head if surplus > 0 else ~head).flatten()
        pick = where[_permutation(int(where.numel()), gen, dev)[:abs(surplus)].long()]
        head[pick] = surplus < 0
        del where, pick
    out_s, out_d = torch.empty_like(s), torch.empty_like(d)
    for src_arr, out in ((s, out_s), (d, out_d)):
        gen_state = gen.get_state()           # the same permutations for both arrays
        first = src_arr[:h][_permutation(h, gen, dev)]
        second = src_arr[h:][_permutation(m - h, gen, dev)]
        if src_arr is s:
            gen.set_state(gen_state)
        used_first = used_second = 0
        for a in range(0, m, _SEGMENT):
            b = min(m, a + _SEGMENT)
            pat = pattern[a:b]
            c = int(pat.sum().item())
            seg = out[a:b]
            seg[pat] = first[used_first:used_first + c]
            seg[~pat] = second[used_second:used_second + (b - a - c)]
            used_first += c
            used_second += b - a - c
        del first, second
    return out_s, out_d
