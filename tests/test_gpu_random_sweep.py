"""Planned runs and plan evaluation on randomly drawn graphs, launch shapes and seeds against the oracle,
element by element: a sweep over what the hand-picked cases fix (graph family, n, k on plans for 16 and 32
partitions, chunk lengths from one tile to several groups of 32 tiles, even and odd, hub degree, column-block
size, pass count, slack, no / partial / complete seed)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2502_17846_amd import binding as B
from paper_2502_17846_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _draw(case):
    rng = np.random.default_rng([2502, case])
    n = int(rng.integers(2000, 120000))
    m = int(n * rng.integers(3, 14))
    kind = int(rng.integers(0, 3))
    if kind == 0:
        g = synth.chung_lu(n=n, m=m, gamma=2.1, cap=float(rng.integers(200, 5000)), seed=int(rng.integers(1 << 30)))
    elif kind == 1:
        g = synth.random_graph_np(n, m, int(rng.integers(1 << 30)), simple=bool(rng.integers(0, 2)))
    else:
        scale = int(np.log2(n))
        g = synth.hub_stress(scale=scale, edge_factor=int(rng.integers(2, 8)), hubs=int(rng.integers(1, 6)),
                             hub_degree=int(min(rng.integers(500, 6000), (1 << scale) // 2)), seed=int(rng.integers(1 << 30)))
    g = synth.to_numpy(g)
    k = int(rng.choice([2, 3, 4, 5, 7, 8, 9, 13, 16, 17, 24, 32]))
    chunk = int(rng.choice([1024, 1500, 2048, 3000, 4096, 10000, 33000, 40000, 70000, 1 << 17]))
    R = int(rng.integers(0, 4))
    slack = float(rng.choice([1.0, 1.02, 1.05, 1.3]))
    hub = int(rng.choice([16, 40, 300, 2048, 8192]))
    cb = int(rng.choice([0, 6, 8, 10, 12]))
    mode = int(rng.integers(0, 3))
    seed = None
    if mode == 1:
        seed = np.where(rng.random(g.n) < 0.3, rng.integers(0, k, g.n), -1).astype(np.int32)
    elif mode == 2:
        seed = rng.integers(0, k, g.n).astype(np.int32)
        slack = max(slack, 1.3)
    unlabelled = float(rng.choice([0.0, 0.2]))
    return g, k, chunk, R, slack, hub, cb, seed, unlabelled, rng


@pytest.mark.parametrize("block", range(6))
def test_random_cases(block):
    ran = 0
    for case in range(block * 10, block * 10 + 10):
        g, k, chunk, R, slack, hub, cb, seed, unlabelled, rng = _draw(case)
        print(f"[case {case}] {g.name[:48]} n={g.n} nnz={g.nnz} k={k} chunk={chunk} R={R} slack={slack} hub={hub} cb={cb} "
              f"seed={'none' if seed is None else 'partial' if (seed < 0).any() else 'complete'}", flush=True)
        try:
            olab, osizes, oest = oracle.partition_seeded(g.rowptr, g.colidx, g.n, k, slack, chunk, R, seed, return_state=True)
        except Exception:
            continue                            # (a seed over the capacity, an estimate beyond 32 bits)
        rp, ci = torch.as_tensor(g.rowptr).to(DEV), torch.as_tensor(g.colidx).to(DEV)
        sd = None if seed is None else torch.as_tensor(seed).to(DEV)
        try:
            plan = B.Plan(rp, ci, g.n, chunk, B.options(col_bits=cb, hub_degree=hub, plan_max_k=32 if k > 16 else 0))
        except B.GremError:
            continue                            # (a geometry the two-phase route does not take)
        with plan:
            if k > plan.max_k:
                continue
            for want_est in (False, True):
                # inside a workspace of exactly the advertised size, with a guard area behind it
                need = plan.call_bytes(k, R, seeded=sd is not None, with_estimates_out=want_est)
                ws = torch.full((need + 65536,), 0xA5, dtype=torch.uint8, device=DEV)
                B.grem_set_workspace(ws[:need])
                try:
                    lab, sizes, est = B.grem_partition_planned(plan, k, slack, R, sd, want_sizes=True, want_estimates=want_est)
                    torch.cuda.synchronize()
                finally:
                    B.grem_set_workspace(None)
                assert bool((ws[need:] == 0xA5).all()), f"case {case}: a write beyond the workspace"
                del ws
                bad = np.nonzero(lab.cpu().numpy() != olab)[0]
                assert bad.size == 0, f"case {case}: {bad.size} labels differ, first {bad[:5]}"
                assert sizes.cpu().numpy().tolist() == osizes.tolist()
                if want_est:
                    assert np.array_equal(est.cpu().numpy().view(np.uint32), oest)
            fl = np.where(rng.random(g.n) < unlabelled, -1, olab).astype(np.int32)
            fl_d = torch.as_tensor(fl).to(DEV)
            counts = B.grem_plan_neighbour_counts(plan, k, fl_d)
            cut = B.grem_plan_edge_cut(plan, k, fl_d)
            torch.cuda.synchronize()
            assert np.array_equal(counts.cpu().numpy().view(np.uint32).astype(np.int64),
                                  oracle.neighbour_counts(g.rowptr, g.colidx, g.n, fl, k))
            assert int(cut.item()) == oracle.edge_cut(g.rowptr, g.colidx, g.n, fl)
        ran += 1
    assert ran >= 5
