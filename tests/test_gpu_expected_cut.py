"""Eq. (1) of Sec. 4.2 on the GPU against its oracle, and the shape of the paper's ablation (Sec. 6.2, Fig. 7)
on a synthetic planted bisection: cuts versus chunk size, refined against fixed greedy decisions, next to the
expected cuts at x and at 2x."""
import numpy as np
import pytest
import torch

import oracle
from paper_2502_17846_amd import binding as B
from paper_2502_17846_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
RTOL = 1e-9     # both sides sum the same hypergeometric tail in double; the kernel's log-domain recurrence and
                # scipy's evaluation differ by rounding of lgamma/exp only (about 1e-13 per term)


def _t(a, dtype=None):
    t = torch.as_tensor(np.ascontiguousarray(a))
    return t.to(device=DEV) if dtype is None else t.to(device=DEV, dtype=dtype)


@pytest.mark.parametrize("x", [0.01, 0.1, 0.5, 1.0])
def test_expected_cut_equals_the_oracle(x):
    for g, lab in ((synth.planted_partition(n=10_000, blocks=2, mean_degree=12.0, seed=0), None),
                   (synth.to_numpy(synth.rmat(15, 16, seed=1)), "random")):
        labels = g.planted.astype(np.int32) if lab is None else np.random.default_rng(3).integers(-1, 2, g.n).astype(np.int32)
        want, want_base = oracle.expected_cut(g.rowptr, g.colidx, g.n, labels, x)
        for rdt in (torch.int64, torch.int32):
            out = B.grem_expected_cut(_t(g.rowptr, rdt), _t(g.colidx), g.n, _t(labels), x)
            torch.cuda.synchronize()
            got, base = out.cpu().numpy().tolist()
            assert base == want_base
            assert abs(got - want) <= RTOL * max(1.0, want), (x, got, want)


def _hub_graph(hub_degree, n, extra_edges, seed):
    """One row of `hub_degree` entries (vertex 0 joined to 1..hub_degree) plus random edges among the other
    vertices; symmetric, loop-free, deduplicated CSR."""
    rng = np.random.default_rng(seed)
    a = rng.integers(1, n, extra_edges)
    b = rng.integers(1, n, extra_edges)
    keep = a != b
    src = np.concatenate([np.zeros(hub_degree, np.int64), np.arange(1, hub_degree + 1), a[keep], b[keep]])
    dst = np.concatenate([np.arange(1, hub_degree + 1), np.zeros(hub_degree, np.int64), b[keep], a[keep]])
    key = np.unique(src * n + dst)
    src, dst = key // n, key % n
    rowptr = np.zeros(n + 1, np.int64)
    np.add.at(rowptr, src + 1, 1)
    return np.cumsum(rowptr), dst.astype(np.int32)


def _hub_case(x, extra_edges):
    """A row of 60,000 entries whose 59,000 labelled neighbours are split so unevenly that the mean of the
    majority count in x * 59,000 draws lies about one standard deviation above half the draws: the hub's
    probability of a wrong decision is then neither 0 nor 1 at any x, and its tail has up to x/2 * 59,000 terms."""
    n, hub, k = 80_000, 60_000, 59_000
    rowptr, colidx = _hub_graph(hub, n, extra_edges, seed=21)
    assert rowptr[1] - rowptr[0] == hub
    delta = int(np.sqrt(k * (1.0 - x) / x)) & ~1           # majority minus minority
    labels = np.random.default_rng(22).integers(0, 2, n).astype(np.int32)
    labels[1:hub + 1] = -1
    labels[1:1 + (k + delta) // 2] = 0
    labels[1 + (k + delta) // 2:1 + k] = 1
    if extra_edges == 0:
        labels[0] = -1            # a pure star with an unlabelled centre: the hub's term is the whole sum
    return n, rowptr, colidx, labels, delta


@pytest.mark.parametrize("x", [0.003, 0.05, 0.5, 0.97])
def test_a_row_of_60000_entries(x):
    for extra in (0, 150_000):
        n, rowptr, colidx, labels, delta = _hub_case(x, extra)
        want, want_base = oracle.expected_cut(rowptr, colidx, n, labels, x)
        if extra == 0:
            # E[C] = minority + delta * q for the one row that counts
            q = (want - want_base) / delta
            print(f"[case] star, x={x}: delta={delta} q={q:.4f}", flush=True)
            assert want_base == (59_000 - delta) // 2 and 0.03 < q < 0.97
        for rdt in (torch.int64, torch.int32):
            out = B.grem_expected_cut(_t(rowptr, rdt), _t(colidx), n, _t(labels), x)
            torch.cuda.synchronize()
            got, base = out.cpu().numpy().tolist()
            assert base == want_base
            assert abs(got - want) <= RTOL * max(1.0, want), (x, extra, got, want)


def test_ablation_shape_on_a_planted_bisection():
    g = synth.planted_partition(n=20_000, blocks=2, mean_degree=12.0, seed=7)
    es = synth.edge_stream(g, seed=8)
    s, d = _t(es.src), _t(es.dst)
    P = B.grem_capacity(g.n, 2, 1.05)
    seed = _t(g.planted.astype(np.int32))
    rp, ci = _t(g.rowptr), _t(g.colidx)
    rows = []
    # from the fraction at which a typical node (12 neighbours) draws one neighbour: below it Eq. (1)'s rounded
    # number of draws is zero and the empty draw counts as a tie, i.e. as a right decision
    for x in (0.05, 0.1, 0.2, 0.4):
        c_size = max(1, int(es.m * x))
        cut = {}
        for mode in (B.EDGE_REFINE, B.EDGE_FIXED):
            parts, _, _ = B.grem_edge_stream_bipartition(s, d, g.n, c_size, P, seed, mode, want_nbr_counts=False)
            cut[mode] = int(B.grem_edge_list_cut(s, d, parts).item()) / es.m
        ex = B.grem_expected_cut(rp, ci, g.n, seed, x).cpu().numpy()[0] / g.nnz
        ex2 = B.grem_expected_cut(rp, ci, g.n, seed, min(1.0, 2 * x)).cpu().numpy()[0] / g.nnz
        rows.append((x, cut[B.EDGE_FIXED], cut[B.EDGE_REFINE], ex, ex2))
        print(f"[result] x={x:.2f}  measured fixed {cut[B.EDGE_FIXED]:.4f} refined {cut[B.EDGE_REFINE]:.4f}   "
              f"Eq.(1) at x {ex:.4f}  at 2x {ex2:.4f}", flush=True)
    for x, fixed, refined, ex, ex2 in rows:
        assert refined <= fixed          # refinement never hurts here, and helps at small chunks (Sec. 6.2)
        assert x > 0.1 or refined < 0.7 * fixed
        assert ex2 <= ex + 1e-12         # a doubled effective chunk size never hurts in expectation (Sec. 4.2)
    # small chunks gain the most from refinement, in theory and in practice
    assert rows[0][1] - rows[0][2] > rows[-1][1] - rows[-1][2]
    assert rows[0][3] - rows[0][4] > rows[-1][3] - rows[-1][4]
    # both measured curves and the expectation fall as chunks grow
    assert rows[0][1] > rows[-1][1] and rows[0][3] > rows[-1][3]
