"""GPU parity: the HIP library against the CPU oracle, element by element, through the C ABI.

Labels, partition sizes and the scaled estimates E must be bit-identical; the cut must be equal."""
import json
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2502_17846_amd import binding as B
from paper_2502_17846_amd import synth

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
DEV = "cuda:0"


def _to_dev(g, rowptr_dtype=None):
    rp = torch.as_tensor(np.asarray(g.rowptr))
    if rowptr_dtype is not None:
        rp = rp.to(rowptr_dtype)
    return rp.to(DEV), torch.as_tensor(np.asarray(g.colidx)).to(DEV)


def _check(g, k, slack, chunk, R, seed=None, rowptr_dtype=None, mode=B.HIST_AUTO, tag="", col_bits=0, hub_degree=2048,
           long_row_degree=0):
    """Runs both sides on the same graph and compares everything."""
    g = synth.to_numpy(g)
    print(f"[case] {tag} {g.name} n={g.n} nnz={g.nnz} k={k} slack={slack} chunk={chunk} R={R} "
          f"seeded={seed is not None} rowptr={rowptr_dtype} mode={mode}", flush=True)
    rp, ci = _to_dev(g, rowptr_dtype)
    seed_d = None if seed is None else torch.as_tensor(seed).to(DEV)
    opts = B.options(mode, col_bits, hub_degree, long_row_degree)
    lab, sizes, est = B.grem_partition_state(rp, ci, g.n, k, slack, chunk, R, seed_d, options=opts)
    cut = B.grem_edge_cut(rp, ci, g.n, lab)
    torch.cuda.synchronize()
    olab, osizes, oest = oracle.partition_seeded(g.rowptr, g.colidx, g.n, k, slack, chunk, R, seed,
                                                 return_state=True)
    lab_h = lab.cpu().numpy()
    bad = np.nonzero(lab_h != olab)[0]
    assert bad.size == 0, f"{bad.size} labels differ, first at v={bad[:5]}: gpu {lab_h[bad[:5]]} oracle {olab[bad[:5]]}"
    assert sizes.cpu().numpy().tolist() == osizes.tolist()
    est_h = est.cpu().numpy().view(np.uint32)
    assert (est_h == oest).all(), f"{(est_h != oest).sum()} estimates differ"
    assert int(cut.item()) == oracle.edge_cut(g.rowptr, g.colidx, g.n, olab)
    assert (np.bincount(lab_h, minlength=k) == osizes).all()
    assert osizes.max() <= B.grem_capacity(g.n, k, slack) == oracle.capacity(g.n, k, slack)
    # the same run asking for labels and sizes only: the library then keeps the estimates in its own, narrower
    # tables and takes other kernels for the hubs and the admission
    lab2, sizes2, _ = B.grem_partition_state(rp, ci, g.n, k, slack, chunk, R, seed_d, want_estimates=False, options=opts)
    torch.cuda.synchronize()
    bad = np.nonzero(lab2.cpu().numpy() != olab)[0]
    assert bad.size == 0, f"labels-only run: {bad.size} labels differ, first at v={bad[:5]}"
    assert sizes2.cpu().numpy().tolist() == osizes.tolist()
    return lab_h


def test_handworked_example():
    with open(os.path.join(GOLDEN, "handworked_6v.json")) as f:
        gj = json.load(f)
    e = np.asarray(gj["edges"])
    rowptr, colidx = synth.csr_from_pairs_np(e[:, 0], e[:, 1], gj["n"])
    g = synth.Graph(rowptr, colidx, gj["n"], colidx.size, len(e), None, "handworked")
    c0, c1 = gj["cases"]
    lab = _check(g, gj["k"], c0["balance_slack"], gj["chunk"], c0["refine_passes"])
    assert lab.tolist() == c0["labels"]
    for r in range(c1["refine_passes"] + 1):
        lab = _check(g, gj["k"], c1["balance_slack"], gj["chunk"], r)
        assert lab.tolist() == c1["labels_after_pass"][r]


@pytest.mark.parametrize("rowptr_dtype", [torch.int32, torch.int64])
def test_planted_partition_config(rowptr_dtype):
    g = synth.planted_partition(seed=0)
    for R in (0, 1, 2):
        _check(g, 4, 1.05, 1024, R, rowptr_dtype=rowptr_dtype, tag="unseeded")
    seed = np.full(g.n, -1, dtype=np.int32)
    seed[:1024] = g.planted[:1024]
    _check(g, 4, 1.05, 1024, 2, seed=seed, rowptr_dtype=rowptr_dtype, tag="seeded")


@pytest.mark.parametrize("gseed", range(6))
def test_small_random_graphs(gseed):
    rng = np.random.default_rng(gseed)
    n = int(rng.integers(1, 700))
    m = int(rng.integers(0, 6 * n))
    g = synth.random_graph_np(n, m, gseed, simple=bool(gseed % 2))
    for k in (1, 2, 3, 7, 16):
        for chunk in (1, 5, 100, 256, 1000):
            for slack, R in ((1.0, 2), (1.05, 1), (1.5, 3)):
                _check(g, k, slack, chunk, R)


@pytest.mark.parametrize("k,slack", [(1, 1.0), (2, 1.05), (4, 1.05), (7, 1.0), (8, 1.3), (200, 1.0), (300, 1.1)])
def test_single_chunk_spill_closed_form(k, slack):
    g = synth.random_graph_np(5000, 20000, 3)
    lab = _check(g, k, slack, g.n + 5, 0)
    P = oracle.capacity(g.n, k, slack)
    v = np.arange(g.n)
    expect = np.zeros(g.n, dtype=np.int64) if k == 1 else np.where(v < P, 0, 1 + (v - P) % max(k - 1, 1))
    assert lab.tolist() == expect.tolist()
    # the largest representable chunk size is the same single chunk
    assert _check(g, k, slack, 2**63 - 1, 1).shape == lab.shape
    if k <= 16:
        assert _check(g, k, slack, 2**63 - 1, 0, mode=B.HIST_SWEEP, hub_degree=20).tolist() == expect.tolist()


@pytest.mark.parametrize("n,k,slack,chunk", [(1000, 4, 1.05, 64), (997, 7, 1.0, 100), (4096, 16, 1.05, 1000),
                                              (300, 300, 1.0, 17), (5000, 64, 1.02, 2048)])
def test_edgeless_graph(n, k, slack, chunk):
    g = synth.Graph(np.zeros(n + 1, dtype=np.int64), np.zeros(0, dtype=np.int32), n, 0, 0, None, "edgeless")
    _check(g, k, slack, chunk, 2)


@pytest.mark.parametrize("k", [2, 5, 16, 17, 32, 33, 63, 64, 100, 128, 129, 255, 256, 300, 1000, 1024, 1025, 3000])
def test_many_k(k):
    g = synth.rmat(13, 16, seed=2, rowptr_dtype=torch.int64)
    _check(g, k, 1.05, 1000, 2)


@pytest.mark.parametrize("k", [2, 16, 64])
def test_forced_global_histograms_match(k):
    g = synth.rmat(12, 16, seed=4, rowptr_dtype=torch.int32)
    _check(g, k, 1.05, 700, 2, mode=B.HIST_GLOBAL)


@pytest.mark.parametrize("k", [1, 2, 3, 8, 13, 16])
@pytest.mark.parametrize("col_bits", [4, 9, 0])
def test_two_phase_path_small(k, col_bits):
    g = synth.rmat(13, 16, seed=3, rowptr_dtype=torch.int64)
    _check(g, k, 1.05, 3000, 2, mode=B.HIST_SWEEP, col_bits=col_bits)                  # no hubs
    _check(g, k, 1.05, 3000, 2, mode=B.HIST_SWEEP, col_bits=col_bits, hub_degree=200)  # some rows are hubs
    _check(g, k, 1.2, 5000, 1, mode=B.HIST_SWEEP, col_bits=col_bits, rowptr_dtype=torch.int32, hub_degree=300)


def test_two_phase_path_seeded_and_edge_cases():
    g = synth.planted_partition(n=6000, blocks=3, seed=2, rowptr_dtype=np.int64)
    rng = np.random.default_rng(0)
    seed = np.where(rng.random(g.n) < 0.3, g.planted, -1).astype(np.int32)
    _check(g, 3, 1.05, 2500, 2, seed=seed, mode=B.HIST_SWEEP, col_bits=6, tag="30% seeded")
    _check(g, 3, 1.05, 2500, 2, seed=seed, mode=B.HIST_SWEEP, col_bits=6, hub_degree=14, tag="30% seeded, hubs")
    _check(g, 3, 1.05, 2500, 0, seed=seed, mode=B.HIST_SWEEP, col_bits=6, tag="seeded R=0")
    # a seed that labels every vertex (no tuple to mark as unassigned): a warm start that is refined
    full = np.random.default_rng(1).integers(0, 3, g.n).astype(np.int32)
    _check(g, 3, 1.1, 2500, 2, seed=full, mode=B.HIST_SWEEP, col_bits=6, tag="every vertex seeded")
    _check(g, 3, 1.1, 2500, 0, seed=full, mode=B.HIST_SWEEP, col_bits=6, hub_degree=14, tag="every vertex seeded, hubs, R=0")
    small = synth.planted_partition(n=1500, blocks=3, seed=4, rowptr_dtype=np.int64)
    _check(small, 4, 1.05, 1, 1, mode=B.HIST_SWEEP, col_bits=5, hub_degree=12, tag="chunk=1")
    _check(small, 5, 1.05, 7, 2, mode=B.HIST_SWEEP, col_bits=4, hub_degree=12, tag="chunk=7")
    _check(g, 16, 1.05, 3000, 2, mode=B.HIST_SWEEP, col_bits=18, tag="largest column block")
    _check(g, 16, 1.05, 3000, 2, mode=B.HIST_SWEEP, hub_degree=40_000, tag="32-bit estimates")
    _check(g, 12, 1.05, 3000, 5, mode=B.HIST_SWEEP, hub_degree=2049, tag="32-bit estimates, R=5")
    _check(g, 12, 1.05, 3000, 4, mode=B.HIST_SWEEP, hub_degree=4096, tag="16-bit estimates at the limit")
    _check(g, 16, 1.0, 2049, 3, mode=B.HIST_SWEEP, col_bits=7, hub_degree=16, tag="odd chunk")
    _check(g, 2, 1.0, 6000, 2, mode=B.HIST_SWEEP, col_bits=7, hub_degree=1, tag="every row a hub")
    e = synth.Graph(np.zeros(5001, dtype=np.int64), np.zeros(0, dtype=np.int32), 5000, 0, 0, None, "edgeless")
    _check(e, 16, 1.02, 2048, 2, mode=B.HIST_SWEEP, col_bits=8)
    h = synth.hub_stress(scale=13, edge_factor=8, hubs=4, hub_degree=5000, seed=0, rowptr_dtype=torch.int32)
    _check(h, 16, 1.1, 4096, 2, mode=B.HIST_SWEEP, col_bits=8)
    _check(h, 16, 1.1, 1500, 2, mode=B.HIST_SWEEP, col_bits=8, hub_degree=150)
    _check(h, 7, 1.1, 8192, 1, mode=B.HIST_SWEEP, col_bits=10, hub_degree=40)


def test_wide_plan_long_even_chunks():
    # chunks of 40 tiles (two groups of 32 in the admission's coarse counts), of even length, on a plan for up to
    # 32 partitions: from the second pass on the admission once took the absent packed label table for present
    g = synth.random_graph_np(110_163, 1_321_956, 90298325, simple=True)
    _check(g, 32, 1.3, 40_000, 1, mode=B.HIST_SWEEP, col_bits=10, tag="wide, 40 tiles")
    _check(g, 20, 1.3, 70_000, 2, mode=B.HIST_SWEEP, col_bits=10, tag="wide, 69 tiles")
    _check(g, 16, 1.3, 70_000, 2, mode=B.HIST_SWEEP, col_bits=10, tag="69 tiles")


@pytest.mark.parametrize("k", [17, 20, 23, 32])
def test_two_phase_path_17_to_32_partitions(k):
    # 8-bit labels in the look-up results, 32 counters per row, eight lanes per vertex in the blend
    g = synth.planted_partition(n=6000, blocks=3, mean_degree=10.0, seed=2)
    _check(g, k, 1.05, 2500, 2, mode=B.HIST_SWEEP, col_bits=9, hub_degree=25, tag="wide")
    _check(g, k, 1.0, 2049, 3, mode=B.HIST_SWEEP, col_bits=7, hub_degree=16, tag="wide, odd chunk")
    _check(g, k, 1.05, 3000, 6, mode=B.HIST_SWEEP, hub_degree=2049, tag="wide, 32-bit estimates")
    rng = np.random.default_rng(k)
    seed = np.where(rng.random(g.n) < 0.3, rng.integers(0, k, g.n), -1).astype(np.int32)
    _check(g, k, 1.1, 2500, 2, seed=seed, mode=B.HIST_SWEEP, col_bits=8, hub_degree=30, tag="wide, seeded")
    full = rng.integers(0, k, g.n).astype(np.int32)
    _check(g, k, 1.4, 2500, 1, seed=full, mode=B.HIST_SWEEP, col_bits=8, hub_degree=30, tag="wide, every vertex seeded")
    r = synth.rmat(15, 16, seed=3, rowptr_dtype=torch.int64)
    _check(r, k, 1.05, 1 << 13, 2, mode=B.HIST_SWEEP, col_bits=11, hub_degree=300, tag="wide, rmat")
    h = synth.hub_stress(scale=14, edge_factor=8, hubs=3, hub_degree=3000, seed=2)
    _check(h, k, 1.05, 3000, 2, mode=B.HIST_SWEEP, col_bits=9, hub_degree=200, tag="wide, hubs")
    # some 160 hubs in the one chunk: the admission kernel that works the hubs out itself takes them in
    # several turns (32 hubs per turn and workgroup, four turns' loads at a time)
    _check(g, k, 1.0, 6000, 2, mode=B.HIST_SWEEP, col_bits=8, hub_degree=17, tag="wide, hubs in the admission")


def test_admission_with_several_hundred_hubs_per_chunk():
    # between 256 and 512 hubs per chunk: the one-launch admission takes them in two turns; slack 1.0 keeps
    # partitions at their capacity, so that ranks decide
    g = synth.planted_partition(n=6000, blocks=3, mean_degree=10.0, seed=5)
    _check(g, 16, 1.0, 3000, 2, mode=B.HIST_SWEEP, col_bits=8, hub_degree=14, tag="many hubs in the admission")
    rng = np.random.default_rng(1)
    seed = np.where(rng.random(g.n) < 0.2, rng.integers(0, 7, g.n), -1).astype(np.int32)
    _check(g, 7, 1.02, 3000, 3, seed=seed, mode=B.HIST_SWEEP, col_bits=7, hub_degree=14, tag="many hubs, seeded")


def test_two_phase_path_big_hub():
    # one row longer than 65535 entries: 16-bit counters would overflow if it were not a hub
    h = synth.hub_stress(scale=17, edge_factor=4, hubs=2, hub_degree=100_000, seed=1, rowptr_dtype=torch.int64)
    _check(h, 16, 1.1, 1 << 15, 2, mode=B.HIST_SWEEP, col_bits=12)


def test_two_phase_path_errors():
    g = synth.random_graph_np(100, 300, 0)
    rp, ci = _to_dev(g)
    with pytest.raises(B.GremError) as e:
        B.grem_partition(rp, ci, g.n, 33, 1.05, 10, 1, options=B.options(B.HIST_SWEEP))
    assert e.value.code == B.ERR_ARG
    with pytest.raises(B.GremError) as e:      # more than 16 partitions need column blocks of at most 2^16 vertices
        B.grem_partition(rp, ci, g.n, 17, 1.05, 10, 1, options=B.options(B.HIST_SWEEP, col_bits=17))
    assert e.value.code == B.ERR_ARG
    for bad in (B.options(histogram_mode=7), B.options(col_bits=3), B.options(col_bits=19), B.options(hub_degree=-1),
                B.options(hub_degree=65536), B.options(long_row_degree=-5)):
        with pytest.raises(B.GremError) as e:
            B.grem_partition(rp, ci, g.n, 4, 1.05, 10, 1, options=bad)
        assert e.value.code == B.ERR_ARG
    bad = B.options()
    bad.reserved[2] = 1
    with pytest.raises(B.GremError) as e:
        B.grem_partition(rp, ci, g.n, 4, 1.05, 10, 1, options=bad)
    assert e.value.code == B.ERR_ARG


def test_rmat_ragged_chunks_and_tiles():
    g = synth.rmat(15, 16, seed=1, rowptr_dtype=torch.int32)
    _check(g, 8, 1.05, 3000, 2)          # chunk not a multiple of any tile
    _check(g, 8, 1.03, g.n, 1)           # one chunk
    _check(g, 32, 1.05, 4097, 1)


def test_hubs():
    g = synth.hub_stress(scale=13, edge_factor=8, hubs=4, hub_degree=5000, seed=0, rowptr_dtype=torch.int32)
    _check(g, 16, 1.1, 1024, 2)
    _check(g, 256, 1.1, 1024, 2)


def test_long_rows_get_a_grid_of_their_own():
    # plain score kernels (histograms in LDS, then in E's rows), long rows split off at several thresholds
    g = synth.hub_stress(scale=13, edge_factor=8, hubs=4, hub_degree=5000, seed=0, rowptr_dtype=torch.int32)
    _check(g, 16, 1.1, 1024, 2, mode=B.HIST_LDS, long_row_degree=1000, tag="4 long rows")
    _check(g, 256, 1.1, 1024, 2, long_row_degree=1000, tag="4 long rows, k=256")
    _check(g, 16, 1.1, 3000, 2, mode=B.HIST_LDS, long_row_degree=40, tag="many long rows")
    _check(g, 200, 1.1, 3000, 3, mode=B.HIST_GLOBAL, long_row_degree=40, rowptr_dtype=torch.int64,
           tag="many long rows, global")
    _check(g, 5, 1.0, 777, 1, mode=B.HIST_LDS, long_row_degree=1, tag="every non-empty row long")
    rng = np.random.default_rng(3)
    seed = np.where(rng.random(g.n) < 0.4, rng.integers(0, 6, g.n), -1).astype(np.int32)
    _check(g, 6, 1.3, 2048, 2, seed=seed, mode=B.HIST_LDS, long_row_degree=64, tag="seeded, long rows")
    # default threshold: two rows of 100,000 entries, many parts each
    h = synth.hub_stress(scale=17, edge_factor=4, hubs=2, hub_degree=100_000, seed=1, rowptr_dtype=torch.int64)
    _check(h, 16, 1.1, 1 << 15, 2, mode=B.HIST_LDS, tag="default threshold")
    _check(h, 300, 1.1, 1 << 15, 1, tag="default threshold, k=300")


def test_seeded_everything_and_partial():
    g = synth.planted_partition(n=3000, blocks=3, seed=2, rowptr_dtype=np.int64)
    seed = g.planted.copy()
    _check(g, 3, 1.05, 500, 2, seed=seed, tag="all seeded")
    rng = np.random.default_rng(0)
    seed = np.where(rng.random(g.n) < 0.3, g.planted, -1).astype(np.int32)
    _check(g, 3, 1.05, 500, 2, seed=seed, tag="30% seeded")


def test_rmat_scale20_config():
    g = synth.rmat(20, 16, seed=0, device=DEV, rowptr_dtype=torch.int32)
    _check(g, 8, 1.05, 65536, 2)


def test_chung_lu_medium():
    g = synth.chung_lu(2_000_000, 28_000_000, seed=0, device=DEV, rowptr_dtype=torch.int64, cap=20_000.0)
    _check(g, 16, 1.05, 1 << 16, 2, mode=B.HIST_LDS)
    _check(g, 16, 1.05, 1 << 16, 2, mode=B.HIST_SWEEP, col_bits=17)


def test_chung_lu_auto_takes_two_phase_path():
    g = synth.chung_lu(6_000_000, 60_000_000, seed=1, device=DEV, rowptr_dtype=torch.int64, cap=30_000.0)
    _check(g, 16, 1.05, 1 << 19, 2)
    # a chunk size that is no power of two (and no multiple of a slice or a column block), fewer partitions
    _check(g, 12, 1.02, 777_777, 1, tag="ragged geometry")
    rng = np.random.default_rng(11)
    seed = np.where(rng.random(g.n) < 0.05, rng.integers(0, 8, g.n), -1).astype(np.int32)
    _check(g, 8, 1.1, 500_000, 1, seed=seed, tag="seeded, two-phase by AUTO")


def test_determinism_and_workspace():
    g = synth.rmat(16, 16, seed=5, device=DEV, rowptr_dtype=torch.int32)
    k, chunk = 16, 5000
    a = B.grem_partition(g.rowptr, g.colidx, g.n, k, 1.05, chunk, 2)
    sweep = B.options(B.HIST_SWEEP, col_bits=10, hub_degree=300)
    small_ws, big_ws = B.grem_workspace_bytes(g.n, k, chunk), B.grem_workspace_bytes_two_phase(g.n, g.nnz, k, chunk, sweep)
    assert 0 < small_ws < big_ws
    ws = torch.empty(big_ws, dtype=torch.uint8, device=DEV)
    B.grem_set_workspace(ws)
    try:
        b = B.grem_partition(g.rowptr, g.colidx, g.n, k, 1.05, chunk, 2)
        c = B.grem_partition(g.rowptr, g.colidx, g.n, k, 1.05, chunk, 2)
        # the two-phase route inside the same workspace, and refused in one that only holds the plain route
        d = B.grem_partition(g.rowptr, g.colidx, g.n, k, 1.05, chunk, 2, options=sweep)
        assert torch.equal(a, d)
        B.grem_set_workspace(ws[:small_ws])
        e_ = B.grem_partition(g.rowptr, g.colidx, g.n, k, 1.05, chunk, 2)
        assert torch.equal(a, e_)
        with pytest.raises(B.GremError) as e:
            B.grem_partition(g.rowptr, g.colidx, g.n, k, 1.05, chunk, 2, options=sweep)
        assert e.value.code == B.ERR_NOMEM
        small = torch.empty(1024, dtype=torch.uint8, device=DEV)
        B.grem_set_workspace(small)
        with pytest.raises(B.GremError) as e:
            B.grem_partition(g.rowptr, g.colidx, g.n, k, 1.05, chunk, 2)
        assert e.value.code == B.ERR_NOMEM
    finally:
        B.grem_set_workspace(None)
    torch.cuda.synchronize()
    assert torch.equal(a, b) and torch.equal(a, c)


def test_errors():
    g = synth.random_graph_np(100, 300, 0)
    rp, ci = _to_dev(g)
    for bad in (dict(k=0), dict(k=B.MAX_K + 1), dict(chunk=0), dict(R=-1), dict(slack=0.99), dict(slack=float("nan"))):
        args = dict(k=4, chunk=10, R=1, slack=1.05)
        args.update(bad)
        with pytest.raises(B.GremError) as e:
            B.grem_partition(rp, ci, g.n, args["k"], args["slack"], args["chunk"], args["R"])
        assert e.value.code == B.ERR_ARG
    with pytest.raises(B.GremError) as e:
        B.grem_partition(rp, ci, g.n, 4, 1.05, 10, 31)
    assert e.value.code == B.ERR_RANGE
    seed = torch.full((g.n,), -1, dtype=torch.int32, device=DEV)
    seed[3] = 4
    with pytest.raises(B.GremError) as e:
        B.grem_partition_seeded(rp, ci, g.n, 4, 1.05, 10, 1, seed)
    assert e.value.code == B.ERR_SEED
    seed[:] = 0
    with pytest.raises(B.GremError) as e:
        B.grem_partition_seeded(rp, ci, g.n, 4, 1.05, 10, 1, seed)
    assert e.value.code == B.ERR_SEED
    # after errors the library still works
    lab = B.grem_partition(rp, ci, g.n, 4, 1.05, 10, 1)
    torch.cuda.synchronize()
    assert lab.cpu().numpy().tolist() == oracle.partition(g.rowptr, g.colidx, g.n, 4, 1.05, 10, 1).tolist()
