"""A fixed labelling evaluated on a plan (grem_plan_neighbour_counts, grem_plan_edge_cut,
grem_plan_expected_cut): cnt_nbrs of Alg. 2 for every vertex at once, the cut of Sec. 1 and Eq. (1) of
Sec. 4.2, each compared with the oracle (counts and cut exactly, Eq. (1) to 1e-9 relative)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2502_17846_amd import binding as B
from paper_2502_17846_amd import synth
from tests.test_gpu_expected_cut import _hub_case

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
RTOL = 1e-9


def _dev(g, rdt=torch.int64):
    g = synth.to_numpy(g)
    return g, torch.as_tensor(g.rowptr).to(device=DEV, dtype=rdt), torch.as_tensor(g.colidx).to(DEV)


def _labels(n, k, none_share, seed):
    rng = np.random.default_rng(seed)
    lab = rng.integers(0, k, n).astype(np.int32)
    if none_share:
        lab[rng.random(n) < none_share] = -1
    return lab


def _check_counts_and_cut(g, plan, k, lab):
    lab_d = torch.as_tensor(lab).to(DEV)
    counts = B.grem_plan_neighbour_counts(plan, k, lab_d)
    cut = B.grem_plan_edge_cut(plan, k, lab_d)
    torch.cuda.synchronize()
    want = oracle.neighbour_counts(g.rowptr, g.colidx, g.n, lab, k)
    got = counts.cpu().numpy().view(np.uint32).astype(np.int64)
    bad = np.nonzero((got != want).any(axis=1))[0]
    assert bad.size == 0, f"{bad.size} rows differ, first {bad[:5]}: {got[bad[:2]]} vs {want[bad[:2]]}"
    assert int(cut.item()) == oracle.edge_cut(g.rowptr, g.colidx, g.n, lab)


@pytest.mark.parametrize("rdt", [torch.int64, torch.int32])
def test_counts_and_cut_with_hubs_and_shares(rdt):
    # hubs (rows of >= 300 entries), a ragged last chunk, several column blocks per chunk
    g, rp, ci = _dev(synth.hub_stress(scale=14, edge_factor=8, hubs=3, hub_degree=3000, seed=2), rdt)
    with B.Plan(rp, ci, g.n, 3000, B.options(col_bits=9, hub_degree=300)) as plan:
        assert B.load().grem_plan_n(plan._h) == g.n
        for k, none_share in ((2, 0.0), (2, 0.3), (3, 0.1), (16, 0.0), (16, 0.5), (1, 0.0), (7, 1.0)):
            print(f"[case] plan counts k={k} unlabelled share {none_share} rowptr {rdt}", flush=True)
            _check_counts_and_cut(g, plan, k, _labels(g.n, k, none_share, 40 + k))
        # the plan serves partition runs as before, and their labels' cut agrees with the CSR walk
        lab = B.grem_partition_planned(plan, 5, 1.05, 1)
        cut = B.grem_plan_edge_cut(plan, 5, lab)
        torch.cuda.synchronize()
        assert int(cut.item()) == int(B.grem_edge_cut(rp, ci, g.n, lab).item())
        with pytest.raises(B.GremError) as e:
            B.grem_plan_neighbour_counts(plan, 4, torch.full((g.n,), 4, dtype=torch.int32, device=DEV))
        assert e.value.code == B.ERR_SEED
        with pytest.raises(B.GremError) as e:
            B.grem_plan_edge_cut(plan, 17, torch.zeros(g.n, dtype=torch.int32, device=DEV))
        assert e.value.code == B.ERR_ARG


def test_counts_and_cut_with_more_than_16_partitions():
    g, rp, ci = _dev(synth.rmat(scale=15, edge_factor=12, seed=9))
    with B.Plan(rp, ci, g.n, 5000, B.options(col_bits=10, hub_degree=200, plan_max_k=32)) as plan:
        for k, none_share in ((32, 0.0), (17, 0.2), (4, 0.0)):
            print(f"[case] plan counts on a plan for k <= 32, k={k} unlabelled share {none_share}", flush=True)
            _check_counts_and_cut(g, plan, k, _labels(g.n, k, none_share, 60 + k))


def test_counts_inside_a_workspace():
    g, rp, ci = _dev(synth.chung_lu(n=60_000, m=420_000, gamma=2.1, cap=5_000.0, seed=4))
    k = 6
    with B.Plan(rp, ci, g.n, 1 << 14) as plan:
        ws = torch.empty(plan.call_bytes(k, 0, seeded=True, with_estimates_out=True) + g.n * k * 4 + 512,
                         dtype=torch.uint8, device=DEV)
        B.grem_set_workspace(ws)
        try:
            _check_counts_and_cut(g, plan, k, _labels(g.n, k, 0.05, 77))
        finally:
            B.grem_set_workspace(None)


@pytest.mark.parametrize("x", [0.01, 0.1, 0.5, 1.0])
def test_expected_cut_on_a_plan_equals_the_oracle(x):
    g, rp, ci = _dev(synth.chung_lu(n=40_000, m=320_000, gamma=2.1, cap=5_000.0, seed=12))
    for none_share in (0.0, 0.15):
        lab = _labels(g.n, 2, none_share, 90)
        want, want_base = oracle.expected_cut(g.rowptr, g.colidx, g.n, lab, x)
        with B.Plan(rp, ci, g.n, 1 << 13, B.options(col_bits=10, hub_degree=100)) as plan:
            out = B.grem_plan_expected_cut(plan, torch.as_tensor(lab).to(DEV), x)
            torch.cuda.synchronize()
            got, base = out.cpu().numpy().tolist()
            assert base == want_base
            assert abs(got - want) <= RTOL * max(1.0, want), (x, none_share, got, want)
            with pytest.raises(B.GremError) as e:
                B.grem_plan_expected_cut(plan, torch.full((g.n,), 2, dtype=torch.int32, device=DEV), x)
            assert e.value.code == B.ERR_SEED


@pytest.mark.parametrize("x", [0.003, 0.5])
def test_expected_cut_on_a_plan_with_a_row_of_60000_entries(x):
    n, rowptr, colidx, labels, delta = _hub_case(x, 150_000)
    want, want_base = oracle.expected_cut(rowptr, colidx, n, labels, x)
    rp = torch.as_tensor(rowptr).to(DEV)
    ci = torch.as_tensor(colidx).to(DEV)
    with B.Plan(rp, ci, n, 1 << 14) as plan:
        out = B.grem_plan_expected_cut(plan, torch.as_tensor(labels).to(DEV), x)
        torch.cuda.synchronize()
        got, base = out.cpu().numpy().tolist()
        assert base == want_base
        assert abs(got - want) <= RTOL * max(1.0, want), (x, got, want)


def test_degenerate_graphs():
    # no entries at all; fewer vertices than a slice of rows, one ragged chunk, loops and repeated entries
    e = synth.Graph(np.zeros(5001, dtype=np.int64), np.zeros(0, dtype=np.int32), 5000, 0, 0, None, "edgeless")
    rp, ci = torch.as_tensor(e.rowptr).to(DEV), torch.zeros(1, dtype=torch.int32, device=DEV)
    with B.Plan(rp, ci, e.n, 2048) as plan:
        lab = _labels(e.n, 3, 0.2, 5)
        counts = B.grem_plan_neighbour_counts(plan, 3, torch.as_tensor(lab).to(DEV))
        cut = B.grem_plan_edge_cut(plan, 3, torch.as_tensor(lab).to(DEV))
        out = B.grem_plan_expected_cut(plan, torch.as_tensor(np.minimum(lab, 1)).to(DEV), 0.5)
        torch.cuda.synchronize()
        assert int(counts.abs().sum()) == 0 and int(cut.item()) == 0 and out.cpu().numpy().tolist() == [0.0, 0.0]
    rng = np.random.default_rng(8)
    n = 37
    deg = rng.integers(0, 6, n)
    rowptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int64)
    colidx = rng.integers(0, n, int(rowptr[-1])).astype(np.int32)
    g = synth.Graph(rowptr, colidx, n, int(rowptr[-1]), 0, None, "tiny multigraph")
    with B.Plan(torch.as_tensor(rowptr).to(DEV), torch.as_tensor(colidx).to(DEV), n, 1 << 20) as plan:
        for k, none_share in ((1, 0.0), (2, 0.3), (16, 0.0)):
            _check_counts_and_cut(g, plan, k, _labels(n, k, none_share, 3 + k))
        lab = _labels(n, 2, 0.2, 1)
        want, want_base = oracle.expected_cut(rowptr, colidx, n, lab, 0.7)
        got, base = B.grem_plan_expected_cut(plan, torch.as_tensor(lab).to(DEV), 0.7).cpu().numpy().tolist()
        assert base == want_base and abs(got - want) <= RTOL * max(1.0, want)
