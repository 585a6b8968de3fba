"""GPU parity of the edge-chunk path (Alg. 1 in the paper's own stream model, two partitions): parts,
sizes, nbr_counts (bit for bit: both sides do the same two IEEE double operations per blend) and the
cut equal the CPU oracle's, through the C ABI."""
import json
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2502_17846_amd import binding as B
from paper_2502_17846_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _t(a, dtype=torch.int32):
    return torch.as_tensor(np.ascontiguousarray(a)).to(device=DEV, dtype=dtype)


def _check(src, dst, n, c_size, P, seed, mode=B.EDGE_REFINE, tag=""):
    print(f"[case] edge stream {tag} n={n} m={len(src)} c_size={c_size} P={P} mode={mode}", flush=True)
    s, d, sd = _t(src), _t(dst), _t(seed)
    parts, sizes, est = B.grem_edge_stream_bipartition(s, d, n, c_size, P, sd, mode)
    cut = B.grem_edge_list_cut(s, d, parts)
    torch.cuda.synchronize()
    oparts, osizes, oest = oracle.edge_stream_bipartition(src, dst, n, c_size, P, seed, mode, return_state=True)
    assert np.array_equal(parts.cpu().numpy(), oparts), tag
    assert sizes.cpu().numpy().tolist() == osizes.tolist(), tag
    assert np.array_equal(est.cpu().numpy().view(np.uint64), oest.view(np.uint64)), tag
    assert int(cut.item()) == oracle.edge_list_cut(src, dst, oparts), tag
    # without the optional outputs
    parts2, _, _ = B.grem_edge_stream_bipartition(s, d, n, c_size, P, sd, mode, want_sizes=False, want_nbr_counts=False)
    torch.cuda.synchronize()
    assert torch.equal(parts, parts2), tag
    return oparts


def test_handworked_examples():
    with open(os.path.join(GOLDEN, "handworked_edge_stream.json")) as f:
        cases = json.load(f)["cases"]
    for c in cases:
        e = np.asarray(c["edges"], dtype=np.int32)
        seed = np.asarray(c["seed_parts"], dtype=np.int32)
        for key, mode in (("refine", B.EDGE_REFINE), ("fixed", B.EDGE_FIXED)):
            if key not in c:
                continue
            parts = _check(e[:, 0], e[:, 1], c["n"], c["c_size"], c["P"], seed, mode, tag=c["name"][:40])
            assert parts.tolist() == c[key]["parts"]


@pytest.mark.parametrize("mode", [B.EDGE_REFINE, B.EDGE_FIXED])
@pytest.mark.parametrize("frac", [0.5, 0.05, 0.003])
def test_planted_bisection(mode, frac):
    g = synth.planted_partition(n=10_000, blocks=2, mean_degree=10.0, seed=0)
    es = synth.edge_stream(g, seed=3)
    P = oracle.capacity(g.n, 2, 1.03)
    _check(es.src, es.dst, g.n, max(1, int(es.m * frac)), P, g.planted.astype(np.int32), mode, tag=f"planted frac={frac}")


@pytest.mark.parametrize("seed_", range(4))
def test_random_multigraphs_with_loops_tight_capacity(seed_):
    # repeated edges, loops, nodes that never occur, capacity exactly n/2 so that partitions fill up,
    # requests are rejected by rank and new nodes are spilled; chunk sizes that leave a ragged tail
    rng = np.random.default_rng(seed_)
    n = int(rng.integers(3_000, 6_000)) * 2
    m = int(rng.integers(20_000, 60_000))
    src = rng.integers(0, n - 100, m).astype(np.int32)
    dst = np.where(rng.random(m) < 0.02, src, rng.integers(0, n - 100, m)).astype(np.int32)
    seed = rng.integers(0, 2, n).astype(np.int32)
    c_size = int(rng.integers(500, 3_000))
    first = np.unique(np.concatenate([src[:c_size], dst[:c_size]]))
    # a balanced seed for the first chunk's nodes
    seed[first] = np.arange(first.size) % 2
    for mode in (B.EDGE_REFINE, B.EDGE_FIXED):
        _check(src, dst, n, c_size, n // 2, seed, mode, tag=f"multigraph seed={seed_}")


def test_many_reappearances_round_the_mean():
    # 12 nodes, thousands of chunks: each node is blended far more often than a double has mantissa
    # bits, so the sums are rounded; the GPU must round exactly as the oracle does
    rng = np.random.default_rng(0)
    n, m = 12, 30_000
    src = rng.integers(0, n, m).astype(np.int32)
    dst = rng.integers(0, n, m).astype(np.int32)
    seed = (np.arange(n) % 2).astype(np.int32)
    _check(src, dst, n, 7, 7, seed, tag="many reappearances")
    _check(src, dst, n, 1, 6, seed, tag="one edge per chunk")


def test_rmat_power_law_stream_spans_many_workgroups():
    g = synth.rmat(18, 8, seed=1)
    es = synth.edge_stream(g, seed=2)
    src, dst = es.src.numpy(), es.dst.numpy()
    n = g.n
    rng = np.random.default_rng(4)
    seed = rng.integers(0, 2, n).astype(np.int32)
    for c_size, slack in ((es.m // 10, 1.05), (es.m // 3 + 1, 1.0), (es.m, 1.2)):
        P = oracle.capacity(n, 2, slack)
        first = np.unique(np.concatenate([src[:c_size], dst[:c_size]]))
        sd = seed.copy()
        sd[first] = np.arange(first.size) % 2
        _check(src, dst, n, c_size, P, sd, tag=f"rmat-18 c_size={c_size}")


def test_errors():
    n = 100
    src = _t(np.arange(50)); dst = _t(np.arange(50) + 50)
    seed = _t(np.zeros(n))
    with pytest.raises(B.GremError) as ei:          # seed overfills partition 0 (P = 50, 100 seeded)
        B.grem_edge_stream_bipartition(src, dst, n, 50, 50, seed)
    assert ei.value.code == B.ERR_SEED
    with pytest.raises(B.GremError) as ei:          # 2P < n
        B.grem_edge_stream_bipartition(src, dst, n, 10, 49, seed)
    assert ei.value.code == B.ERR_ARG
    bad = _t(np.arange(50) + 51)                     # an endpoint equal to n
    with pytest.raises(B.GremError) as ei:
        B.grem_edge_stream_bipartition(src, bad, n, 10, 60, seed)
    assert ei.value.code == B.ERR_ARG
    seed2 = _t(np.full(n, -1))
    with pytest.raises(B.GremError) as ei:          # first chunk's nodes carry no seed label
        B.grem_edge_stream_bipartition(src, dst, n, 10, 60, seed2)
    assert ei.value.code == B.ERR_SEED
    with pytest.raises(B.GremError) as ei:
        B.grem_edge_stream_bipartition(src, dst, n, 10, 60, seed, mode=7)
    assert ei.value.code == B.ERR_ARG
    # the library is still usable afterwards
    ok = _t(np.arange(n) % 2)
    parts, sizes, _ = B.grem_edge_stream_bipartition(src, dst, n, 10, 60, ok)
    torch.cuda.synchronize()
    assert int(sizes.sum()) == 100 and int(parts.min()) >= 0


# ---------------------------------------------------------------------------------------------
# recursive bisection
# ---------------------------------------------------------------------------------------------

def _check_rb(src, dst, n, levels, chunks, slack, bits, mode=B.EDGE_REFINE, tag=""):
    print(f"[case] recursive bisection {tag} n={n} m={len(src)} levels={levels} chunks={chunks} slack={slack}", flush=True)
    lab = B.grem_recursive_bisection(_t(src), _t(dst), n, levels, chunks, slack, _t(bits).reshape(-1), mode)
    torch.cuda.synchronize()
    olab = oracle.recursive_bisection(src, dst, n, levels, chunks, slack, bits, mode)
    assert np.array_equal(lab.cpu().numpy(), olab), tag
    return olab


def test_recursive_bisection_planted_blocks():
    g = synth.planted_partition(n=10_000, blocks=4, mean_degree=12.0, seed=5)
    es = synth.edge_stream(g, seed=6)
    bits = np.stack([g.planted >> 1, g.planted & 1]).astype(np.int32)
    for mode in (B.EDGE_REFINE, B.EDGE_FIXED):
        lab = _check_rb(es.src, es.dst, g.n, 2, 20, 1.05, bits, mode, tag="planted 4 blocks")
        assert np.bincount(lab, minlength=4).max() <= oracle.capacity(oracle.capacity(g.n, 2, 1.05), 2, 1.05)


@pytest.mark.parametrize("seed_", range(3))
def test_recursive_bisection_random_multigraphs(seed_):
    # loops, repeated edges, nodes in no edge (placed by size), groups that run out of inside edges
    rng = np.random.default_rng(100 + seed_)
    n = int(rng.integers(2_000, 9_000))
    m = int(rng.integers(n, 6 * n))
    src = rng.integers(0, n - 50, m).astype(np.int32)
    dst = np.where(rng.random(m) < 0.02, src, rng.integers(0, n - 50, m)).astype(np.int32)
    levels = int(rng.integers(1, 6))
    bits = np.stack([(np.arange(n) >> l) & 1 for l in range(levels)]).astype(np.int32)
    _check_rb(src, dst, n, levels, int(rng.integers(1, 30)), 1.1, bits, tag=f"multigraph {seed_}")


def test_recursive_bisection_sparse_graph_deep_levels():
    # fewer edges than nodes: deep levels meet groups without inside edges and empty chunks' tails
    rng = np.random.default_rng(7)
    n, m = 3_000, 2_000
    src = rng.integers(0, n, m).astype(np.int32)
    dst = rng.integers(0, n, m).astype(np.int32)
    bits = np.stack([(np.arange(n) >> l) & 1 for l in range(7)]).astype(np.int32)
    lab = _check_rb(src, dst, n, 7, 4, 1.3, bits, tag="sparse deep")
    assert lab.max() < 128


def test_recursive_bisection_rmat():
    g = synth.rmat(16, 8, seed=3)
    es = synth.edge_stream(g, seed=4)
    src, dst = es.src.numpy(), es.dst.numpy()
    bits = np.stack([(np.arange(g.n) >> l) & 1 for l in range(4)]).astype(np.int32)
    _check_rb(src, dst, g.n, 4, 25, 1.05, bits, tag="rmat-16 k=16")


def test_recursive_bisection_chung_lu_million_nodes():
    # 1.4M nodes, 20M edges, 16 partitions: every level spans many workgroups of every kernel; the oracle
    # needs about a quarter of a minute
    g = synth.chung_lu(1_387_500, 20_000_000, seed=2, device=DEV, rowptr_dtype=torch.int64, cap=20_000.0)
    es = synth.edge_stream(g, seed=3)
    src, dst = es.src.cpu().numpy(), es.dst.cpu().numpy()
    bits = np.stack([(np.arange(g.n) >> l) & 1 for l in range(4)]).astype(np.int32)
    lab = _check_rb(src, dst, g.n, 4, 50, 1.05 ** 0.25, bits, tag="chung-lu 1.4M k=16")
    assert np.bincount(lab, minlength=16).max() <= 1.05 * g.n / 16 + 16


def test_degenerate_streams():
    # one node with a loop; a stream of identical edges; only loops; more chunks than distinct nodes
    _check(np.array([0], np.int32), np.array([0], np.int32), 1, 1, 1, np.array([1], np.int32), tag="single loop")
    _check(np.full(500, 3, np.int32), np.full(500, 68, np.int32), 70, 7, 35, (np.arange(70) % 2).astype(np.int32),
           tag="identical edges")
    ids = (np.arange(300) % 65).astype(np.int32)
    _check(ids, ids, 65, 10, 33, (np.arange(65) % 2).astype(np.int32), tag="only loops")
    _check(ids, ids[::-1].copy(), 65, 1, 33, (np.arange(65) % 2).astype(np.int32), mode=B.EDGE_FIXED, tag="one edge per chunk, fixed")
    lab = _check_rb(ids, ids[::-1].copy(), 65, 3, 2, 1.5, np.stack([(np.arange(65) >> l) & 1 for l in range(3)]).astype(np.int32),
                    tag="tiny recursion")
    assert lab.max() < 8
