"""GPU parity of the edge-bucket build (Sec. 3, storage layer): grouped edges and bucket offsets equal the
CPU oracle's (a stable sort by (label[src], label[dst])), through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2502_17846_amd import binding as B
from paper_2502_17846_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _t(a, dtype=torch.int32):
    return torch.as_tensor(np.ascontiguousarray(a)).to(device=DEV, dtype=dtype)


def _check(src, dst, n, lab, k, tag=""):
    print(f"[case] edge buckets {tag} n={n} m={len(src)} k={k}", flush=True)
    os_, od_, off = B.grem_edge_buckets(_t(src), _t(dst), n, _t(lab), k)
    torch.cuda.synchronize()
    ws, wd, woff = oracle.edge_buckets(src, dst, lab, k)
    assert off.cpu().numpy().tolist() == woff.tolist(), tag
    assert np.array_equal(os_.cpu().numpy(), ws), tag
    assert np.array_equal(od_.cpu().numpy(), wd), tag


@pytest.mark.parametrize("k", [1, 2, 3, 16, 17, 32, 33, 64, 128])
def test_random_edges_all_bucket_counts(k):
    rng = np.random.default_rng(k)
    n, m = 5_000, 70_001                       # several tiles and a ragged tail
    src = rng.integers(0, n, m).astype(np.int32)
    dst = rng.integers(0, n, m).astype(np.int32)
    lab = rng.integers(0, k, n).astype(np.int32)
    _check(src, dst, n, lab, k, tag="random")


def test_tiny_and_skewed():
    # fewer edges than a wave; all edges in one bucket; every edge in its own step position
    _check(np.array([3, 1, 2], np.int32), np.array([0, 2, 2], np.int32), 4, np.array([1, 0, 1, 0], np.int32), 2, "tiny")
    rng = np.random.default_rng(0)
    n, m = 1000, 20_000
    src = rng.integers(0, n, m).astype(np.int32)
    dst = rng.integers(0, n, m).astype(np.int32)
    _check(src, dst, n, np.full(n, 5, np.int32), 8, "one bucket")
    lab = np.where(np.arange(n) < 10, 0, 7).astype(np.int32)        # two heavy buckets, two rare ones
    _check(src, dst, n, lab, 8, "skewed")


def test_partitioned_graph_buckets():
    # labels from the partitioner itself, 16 partitions of an R-MAT stream (1M edges, many tiles)
    g = synth.rmat(17, 8, seed=5)
    es = synth.edge_stream(g, seed=6)
    src, dst = es.src.numpy(), es.dst.numpy()
    rp, ci = torch.as_tensor(g.rowptr).to(DEV), torch.as_tensor(g.colidx).to(DEV)
    lab = B.grem_partition(rp, ci, g.n, 16, 1.05, 1 << 14, 1)
    torch.cuda.synchronize()
    _check(src, dst, g.n, lab.cpu().numpy(), 16, "rmat-17 k=16")
    # diagonal buckets hold the uncut edges
    _, _, off = B.grem_edge_buckets(_t(src), _t(dst), g.n, lab, 16)
    cut = int(B.grem_edge_list_cut(_t(src), _t(dst), lab).item())
    sizes = (off[1:] - off[:-1]).reshape(16, 16)
    assert int(sizes.sum() - sizes.diag().sum()) == cut


def test_many_buckets_long_stream_takes_larger_tiles():
    # 16,384 buckets and 40M edges: tiles grow beyond 4,096 edges so that the tile histograms stay within their
    # limit, every workgroup walks its tile in many steps with 64 KB of LDS cursors
    rng = np.random.default_rng(5)
    n, m, k = 200_000, 40_000_000, 128
    src = rng.integers(0, n, m).astype(np.int32)
    dst = rng.integers(0, n, m).astype(np.int32)
    lab = rng.integers(0, k, n).astype(np.int32)
    _check(src, dst, n, lab, k, tag="k=128 long")


def test_errors():
    src, dst = _t(np.arange(10)), _t(np.arange(10)[::-1].copy())
    lab = _t(np.arange(10) % 3)
    with pytest.raises(B.GremError) as ei:               # a label equal to k
        B.grem_edge_buckets(src, dst, 10, lab, 2)
    assert ei.value.code == B.ERR_ARG
    with pytest.raises(B.GremError) as ei:               # k above the limit
        B.grem_edge_buckets(src, dst, 10, lab, 129)
    assert ei.value.code == B.ERR_ARG
    with pytest.raises(B.GremError) as ei:               # endpoint out of range
        B.grem_edge_buckets(src, dst, 9, lab, 3)
    assert ei.value.code == B.ERR_ARG
    os_, od_, off = B.grem_edge_buckets(src, dst, 10, lab, 3)
    torch.cuda.synchronize()
    assert int(off[-1]) == 10
