"""ctypes access to the GREM CPU oracles (``grem_oracle.c``: chunks of CSR rows, k-way;
``grem_edge_oracle.c``: chunks of an edge list, two partitions).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py``.  The GPU package never imports this module and this module
never imports the GPU package.  All arrays are host numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "grem_oracle.c")
_SRC_EDGE = os.path.join(_HERE, "grem_edge_oracle.c")
_LIB = os.path.join(_HERE, "libgrem_oracle.so")

OK = 0
ERR_ARG, ERR_NOMEM, ERR_RANGE, ERR_SEED, ERR_INTERNAL = -1, -2, -3, -4, -5


class OracleError(RuntimeError):
    def __init__(self, code: int):
        super().__init__(f"grem oracle returned {code}")
        self.code = code


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, single thread, no contraction of a*b+c)."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_EDGE))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, _SRC_EDGE, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_LIB)
    i64p, i32p, u32p = (ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int32),
                        ctypes.POINTER(ctypes.c_uint32))
    lib.grem_oracle_capacity.restype = ctypes.c_int64
    lib.grem_oracle_capacity.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_double]
    lib.grem_oracle_create.restype = ctypes.c_void_p
    lib.grem_oracle_create.argtypes = [i64p, i32p, ctypes.c_int64, ctypes.c_int32, ctypes.c_double,
                                       ctypes.c_int64, ctypes.c_int32, i32p,
                                       ctypes.POINTER(ctypes.c_int)]
    lib.grem_oracle_destroy.restype = None
    lib.grem_oracle_destroy.argtypes = [ctypes.c_void_p]
    lib.grem_oracle_step.restype = ctypes.c_int
    lib.grem_oracle_step.argtypes = [ctypes.c_void_p]
    for name, rt in (("grem_oracle_get_capacity", ctypes.c_int64), ("grem_oracle_get_pass", ctypes.c_int32),
                     ("grem_oracle_get_next_chunk", ctypes.c_int64), ("grem_oracle_labels", i32p),
                     ("grem_oracle_sizes", i64p), ("grem_oracle_estimates", u32p)):
        getattr(lib, name).restype = rt
        getattr(lib, name).argtypes = [ctypes.c_void_p]
    lib.grem_oracle_partition_seeded.restype = ctypes.c_int
    lib.grem_oracle_partition_seeded.argtypes = [i64p, i32p, ctypes.c_int64, ctypes.c_int32,
                                                 ctypes.c_double, ctypes.c_int64, ctypes.c_int32,
                                                 i32p, i32p, i64p, u32p]
    lib.grem_oracle_edge_cut.restype = ctypes.c_int64
    lib.grem_oracle_edge_cut.argtypes = [i64p, i32p, ctypes.c_int64, i32p]
    f64p = ctypes.POINTER(ctypes.c_double)
    lib.grem_edge_oracle_create.restype = ctypes.c_void_p
    lib.grem_edge_oracle_create.argtypes = [i32p, i32p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                            ctypes.c_int64, i32p, ctypes.c_int32,
                                            ctypes.POINTER(ctypes.c_int)]
    lib.grem_edge_oracle_destroy.restype = None
    lib.grem_edge_oracle_destroy.argtypes = [ctypes.c_void_p]
    lib.grem_edge_oracle_step.restype = ctypes.c_int
    lib.grem_edge_oracle_step.argtypes = [ctypes.c_void_p]
    for name, rt in (("grem_edge_oracle_parts", i32p), ("grem_edge_oracle_sizes", i64p),
                     ("grem_edge_oracle_nbr_counts", f64p), ("grem_edge_oracle_next_chunk", ctypes.c_int64),
                     ("grem_edge_oracle_chunk_count", ctypes.c_int64)):
        getattr(lib, name).restype = rt
        getattr(lib, name).argtypes = [ctypes.c_void_p]
    lib.grem_edge_oracle_last_nodes.restype = ctypes.c_int64
    lib.grem_edge_oracle_last_nodes.argtypes = [ctypes.c_void_p, ctypes.POINTER(i32p), ctypes.POINTER(i64p),
                                                ctypes.POINTER(i32p)]
    lib.grem_edge_oracle_run.restype = ctypes.c_int
    lib.grem_edge_oracle_run.argtypes = [i32p, i32p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                         ctypes.c_int64, i32p, ctypes.c_int32, i32p, i64p, f64p]
    lib.grem_edge_oracle_cut.restype = ctypes.c_int64
    lib.grem_edge_oracle_cut.argtypes = [i32p, i32p, ctypes.c_int64, i32p]
    _lib = lib
    return lib


def _p(arr, ct):
    return None if arr is None else arr.ctypes.data_as(ctypes.POINTER(ct))


def _csr(rowptr, colidx):
    rp = np.ascontiguousarray(rowptr, dtype=np.int64)
    ci = np.ascontiguousarray(colidx, dtype=np.int32)
    return rp, ci


def capacity(n: int, k: int, balance_slack: float) -> int:
    return int(_load().grem_oracle_capacity(n, k, balance_slack))


def partition_seeded(rowptr, colidx, n, k, balance_slack, chunk, refine_passes, seed_labels=None,
                     return_state: bool = False):
    """Labels (int32[n]) of the whole run; with ``return_state`` also sizes (int64[k]) and the
    scaled estimates E (uint32[n,k])."""
    lib = _load()
    rp, ci = _csr(rowptr, colidx)
    seed = None if seed_labels is None else np.ascontiguousarray(seed_labels, dtype=np.int32)
    labels = np.empty(n, dtype=np.int32)
    sizes = np.empty(k, dtype=np.int64) if return_state else None
    est = np.empty((n, k), dtype=np.uint32) if return_state else None
    rc = lib.grem_oracle_partition_seeded(_p(rp, ctypes.c_int64), _p(ci, ctypes.c_int32), n, k,
                                          float(balance_slack), chunk, refine_passes,
                                          _p(seed, ctypes.c_int32), _p(labels, ctypes.c_int32),
                                          _p(sizes, ctypes.c_int64), _p(est, ctypes.c_uint32))
    if rc != OK:
        raise OracleError(rc)
    if return_state:
        return labels, sizes, est
    return labels


def partition(rowptr, colidx, n, k, balance_slack, chunk, refine_passes):
    return partition_seeded(rowptr, colidx, n, k, balance_slack, chunk, refine_passes, None)


def edge_cut(rowptr, colidx, n, labels) -> int:
    rp, ci = _csr(rowptr, colidx)
    lab = np.ascontiguousarray(labels, dtype=np.int32)
    return int(_load().grem_oracle_edge_cut(_p(rp, ctypes.c_int64), _p(ci, ctypes.c_int32), n,
                                            _p(lab, ctypes.c_int32)))


def neighbour_counts(rowptr, colidx, n, labels, k):
    """cnt_nbrs (Alg. 2) of every vertex under a fixed labelling: out[v, j] = number of CSR entries (v, u)
    with labels[u] == j; entries whose column has no label (-1) are in no count."""
    rp, ci = _csr(rowptr, colidx)
    lab = np.asarray(labels).astype(np.int64)
    rows = np.repeat(np.arange(n, dtype=np.int64), np.diff(rp))
    nl = lab[ci]
    have = nl >= 0
    flat = np.bincount(rows[have] * k + nl[have], minlength=n * k)
    return flat.reshape(n, k).astype(np.int64)


class Stepper:
    """The run one chunk at a time, for tests that look at the state between chunks and for the
    bounded CPU-baseline sample."""

    def __init__(self, rowptr, colidx, n, k, balance_slack, chunk, refine_passes, seed_labels=None):
        self._lib = _load()
        self._rp, self._ci = _csr(rowptr, colidx)   # keep alive: the state borrows them
        self.n, self.k = n, k
        seed = None if seed_labels is None else np.ascontiguousarray(seed_labels, dtype=np.int32)
        status = ctypes.c_int(0)
        self._h = self._lib.grem_oracle_create(_p(self._rp, ctypes.c_int64), _p(self._ci, ctypes.c_int32),
                                               n, k, float(balance_slack), chunk, refine_passes,
                                               _p(seed, ctypes.c_int32), ctypes.byref(status))
        if not self._h:
            raise OracleError(status.value)

    def step(self) -> bool:
        rc = self._lib.grem_oracle_step(self._h)
        if rc < 0:
            raise OracleError(rc)
        return rc == 1

    @property
    def capacity(self) -> int:
        return int(self._lib.grem_oracle_get_capacity(self._h))

    @property
    def position(self):
        """(pass, chunk) of the next step."""
        return int(self._lib.grem_oracle_get_pass(self._h)), int(self._lib.grem_oracle_get_next_chunk(self._h))

    def labels(self) -> np.ndarray:
        return np.ctypeslib.as_array(self._lib.grem_oracle_labels(self._h), shape=(self.n,)).copy()

    def sizes(self) -> np.ndarray:
        return np.ctypeslib.as_array(self._lib.grem_oracle_sizes(self._h), shape=(self.k,)).copy()

    def estimates(self) -> np.ndarray:
        return np.ctypeslib.as_array(self._lib.grem_oracle_estimates(self._h), shape=(self.n, self.k)).copy()

    def close(self):
        if self._h:
            self._lib.grem_oracle_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# --------------------------------------------------------------------------------------------
# chunks of an edge list, two partitions (Alg. 1 in the paper's own stream model)
# --------------------------------------------------------------------------------------------

EDGE_REFINE, EDGE_FIXED = 0, 1


def _edges(src, dst):
    return np.ascontiguousarray(src, dtype=np.int32), np.ascontiguousarray(dst, dtype=np.int32)


def edge_stream_bipartition(src, dst, n, c_size, P, seed_parts, mode=EDGE_REFINE, return_state: bool = False):
    """parts (int32[n], -1 for nodes in no edge); with ``return_state`` also sizes (int64[2]) and
    nbr_counts (float64[n,2])."""
    lib = _load()
    s, d = _edges(src, dst)
    seed = np.ascontiguousarray(seed_parts, dtype=np.int32)
    parts = np.empty(n, dtype=np.int32)
    sizes = np.empty(2, dtype=np.int64) if return_state else None
    est = np.empty((n, 2), dtype=np.float64) if return_state else None
    rc = lib.grem_edge_oracle_run(_p(s, ctypes.c_int32), _p(d, ctypes.c_int32), s.size, n, c_size, P,
                                  _p(seed, ctypes.c_int32), mode, _p(parts, ctypes.c_int32),
                                  _p(sizes, ctypes.c_int64), _p(est, ctypes.c_double))
    if rc != OK:
        raise OracleError(rc)
    if return_state:
        return parts, sizes, est
    return parts


def edge_list_cut(src, dst, parts) -> int:
    s, d = _edges(src, dst)
    lab = np.ascontiguousarray(parts, dtype=np.int32)
    return int(_load().grem_edge_oracle_cut(_p(s, ctypes.c_int32), _p(d, ctypes.c_int32), s.size,
                                            _p(lab, ctypes.c_int32)))


class EdgeStepper:
    """The edge-chunk run one chunk at a time."""

    def __init__(self, src, dst, n, c_size, P, seed_parts, mode=EDGE_REFINE):
        self._lib = _load()
        self._s, self._d = _edges(src, dst)           # keep alive: the state borrows them
        self._seed = np.ascontiguousarray(seed_parts, dtype=np.int32)
        self.n = n
        status = ctypes.c_int(0)
        self._h = self._lib.grem_edge_oracle_create(_p(self._s, ctypes.c_int32), _p(self._d, ctypes.c_int32),
                                                    self._s.size, n, c_size, P,
                                                    _p(self._seed, ctypes.c_int32), mode, ctypes.byref(status))
        if not self._h:
            raise OracleError(status.value)

    def step(self) -> bool:
        rc = self._lib.grem_edge_oracle_step(self._h)
        if rc < 0:
            raise OracleError(rc)
        return rc == 1

    @property
    def next_chunk(self) -> int:
        return int(self._lib.grem_edge_oracle_next_chunk(self._h))

    @property
    def chunk_count(self) -> int:
        return int(self._lib.grem_edge_oracle_chunk_count(self._h))

    def parts(self) -> np.ndarray:
        return np.ctypeslib.as_array(self._lib.grem_edge_oracle_parts(self._h), shape=(self.n,)).copy()

    def sizes(self) -> np.ndarray:
        return np.ctypeslib.as_array(self._lib.grem_edge_oracle_sizes(self._h), shape=(2,)).copy()

    def nbr_counts(self) -> np.ndarray:
        return np.ctypeslib.as_array(self._lib.grem_edge_oracle_nbr_counts(self._h), shape=(self.n, 2)).copy()

    def last_chunk(self):
        """(nodes, fresh counts [c,2], proposals; -2 = not evaluated) of the chunk just processed."""
        i32p, i64p = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)
        nodes, fresh, prop = i32p(), i64p(), i32p()
        c = int(self._lib.grem_edge_oracle_last_nodes(self._h, ctypes.byref(nodes), ctypes.byref(fresh),
                                                      ctypes.byref(prop)))
        if c == 0:
            return np.empty(0, np.int32), np.empty((0, 2), np.int64), np.empty(0, np.int32)
        return (np.ctypeslib.as_array(nodes, shape=(c,)).copy(),
                np.ctypeslib.as_array(fresh, shape=(c, 2)).copy(),
                np.ctypeslib.as_array(prop, shape=(c,)).copy())

    def close(self):
        if self._h:
            self._lib.grem_edge_oracle_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# --------------------------------------------------------------------------------------------
# recursive bisection (Sec. 4.1: more than two partitions by re-partitioning each part in two)
# --------------------------------------------------------------------------------------------

def recursive_bisection(src, dst, n, levels, chunks, balance_slack, seed_bits, mode=EDGE_REFINE,
                        return_levels: bool = False):
    """Labels in [0, 2^levels) for all n nodes.

    Every node starts in group 0.  At each level every group g (ascending) is split in two by the
    edge-chunk procedure run on the group's own subgraph: its nodes renumbered 0..nv-1 in ascending
    id, the edges of the stream with both ends in the group, in stream order, in ceil(m_g / chunks)-edge
    chunks, capacity P = capacity(nv, 2, balance_slack), first chunk seeded with
    seed_bits[level] of its nodes (seed_bits: levels x n, the seed algorithm's answer at each level).  Nodes of the group that no such edge touches are then placed one by one, ascending id,
    in the currently smaller half (0 on a tie).  A node of group g in half b moves to group 2g + b."""
    src = np.ascontiguousarray(src, dtype=np.int32)
    dst = np.ascontiguousarray(dst, dtype=np.int32)
    seed_bits = np.ascontiguousarray(seed_bits, dtype=np.int32).reshape(levels, n)
    label = np.zeros(n, dtype=np.int32)
    history = []
    for level in range(levels):
        nxt = np.empty(n, dtype=np.int32)
        for g in range(1 << level):
            members = np.nonzero(label == g)[0]
            nv = members.size
            if nv == 0:
                continue
            local = np.full(n, -1, dtype=np.int64)
            local[members] = np.arange(nv)
            inside = (label[src] == g) & (label[dst] == g)
            s, d = local[src[inside]].astype(np.int32), local[dst[inside]].astype(np.int32)
            parts = np.full(nv, -1, dtype=np.int32)
            sizes = [0, 0]
            if s.size > 0:
                c_size = (s.size + chunks - 1) // chunks
                P = capacity(nv, 2, balance_slack)
                parts, sz, _ = edge_stream_bipartition(s, d, nv, c_size, P, seed_bits[level][members], mode,
                                                       return_state=True)
                sizes = [int(sz[0]), int(sz[1])]
            for i in np.nonzero(parts < 0)[0]:
                t = 1 if sizes[1] < sizes[0] else 0
                parts[i] = t
                sizes[t] += 1
            nxt[members] = 2 * g + parts
        label = nxt
        history.append(label.copy())
    if return_levels:
        return label, history
    return label


# --------------------------------------------------------------------------------------------
# edge buckets (Sec. 3, storage layer: bucket (i, j) holds the edges from partition i to j)
# --------------------------------------------------------------------------------------------

def edge_buckets(src, dst, labels, k):
    """(out_src, out_dst, offsets): the edges grouped by (labels[src], labels[dst]) in the order of
    i*k + j, each bucket keeping the stream order; offsets has k*k+1 entries (int64)."""
    src = np.ascontiguousarray(src, dtype=np.int32)
    dst = np.ascontiguousarray(dst, dtype=np.int32)
    lab = np.asarray(labels).astype(np.int64)
    if lab.size and (lab[src].min() < 0 or lab[src].max() >= k or lab[dst].min() < 0 or lab[dst].max() >= k):
        raise OracleError(ERR_ARG)
    key = lab[src] * k + lab[dst]
    order = np.argsort(key, kind="stable")
    offsets = np.zeros(k * k + 1, dtype=np.int64)
    np.cumsum(np.bincount(key, minlength=k * k), out=offsets[1:])
    return src[order], dst[order], offsets


# --------------------------------------------------------------------------------------------
# expected number of edge cuts of fixed greedy decisions (Sec. 4.2, Eq. (1))
# --------------------------------------------------------------------------------------------

def expected_cut(rowptr, colidx, n, labels, x):
    """Eq. (1) for a two-way labelling: sum over nodes i of
    (k_i - k0_i) * (1 - q_i) + k0_i * q_i, with k_i the node's labelled neighbours, k0_i those in the
    partition that holds more of them, and q_i = Pr(K < d_i / 2) for K ~ Hypergeometric(population k_i,
    successes k0_i, draws d_i), d_i = floor(k_i * x + 0.5) (the paper's k*x draws, made an integer).
    Also returns sum_i (k_i - k0_i), the value at x = 1.  Every edge is seen from both its ends."""
    from scipy.stats import hypergeom
    rp, ci = _csr(rowptr, colidx)
    lab = np.asarray(labels)
    deg_rows = np.repeat(np.arange(n), np.diff(rp))
    nl = lab[ci]
    c0 = np.bincount(deg_rows[nl == 0], minlength=n).astype(np.int64)
    c1 = np.bincount(deg_rows[nl == 1], minlength=n).astype(np.int64)
    k = c0 + c1
    k0 = np.maximum(c0, c1)
    d = np.floor(k.astype(np.float64) * float(x) + 0.5).astype(np.int64)
    d = np.minimum(d, k)
    # K < d/2  <=>  K <= ceil(d/2) - 1
    q = hypergeom.cdf((d + 1) // 2 - 1, k, k0, d)
    q = np.where(k > 0, q, 0.0)
    total = np.sum((k - k0) * (1.0 - q) + k0 * q)
    return float(total), int(np.sum(k - k0))
