"""Plans (the re-laid-out copy of a graph kept for several runs, grem_plan_*), and concurrent calls on
distinct streams.  Every run is compared with the oracle element by element."""
import numpy as np
import pytest
import torch

import oracle
from paper_2502_17846_amd import binding as B
from paper_2502_17846_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dev(g, rdt=torch.int64):
    g = synth.to_numpy(g)
    return g, torch.as_tensor(g.rowptr).to(device=DEV, dtype=rdt), torch.as_tensor(g.colidx).to(DEV)


def _same_as_oracle(g, out, k, slack, chunk, R, seed=None):
    lab, sizes, est = out
    olab, osizes, oest = oracle.partition_seeded(g.rowptr, g.colidx, g.n, k, slack, chunk, R, seed, return_state=True)
    bad = np.nonzero(lab.cpu().numpy() != olab)[0]
    assert bad.size == 0, f"{bad.size} labels differ, first at {bad[:5]}"
    assert sizes.cpu().numpy().tolist() == osizes.tolist()
    assert np.array_equal(est.cpu().numpy().view(np.uint32), oest)


@pytest.mark.parametrize("rdt", [torch.int64, torch.int32])
def test_one_plan_many_runs(rdt):
    # hubs (rows of >= 300 entries here), ragged last chunk, several column blocks per chunk
    g, rp, ci = _dev(synth.hub_stress(scale=14, edge_factor=8, hubs=3, hub_degree=3000, seed=2), rdt)
    chunk = 3000
    rng = np.random.default_rng(5)
    seed = np.where(rng.random(g.n) < 0.2, rng.integers(0, 3, g.n), -1).astype(np.int32)
    with B.Plan(rp, ci, g.n, chunk, B.options(col_bits=9, hub_degree=300)) as plan:
        assert plan.device_bytes > 5 * g.nnz and plan.max_k == 16
        assert plan.call_bytes(17, 1) == 0 and plan.call_bytes(16, 2) > g.n * 33
        # runs inside a workspace of the size the plan asks for
        ws = torch.empty(plan.call_bytes(3, 2, seeded=True), dtype=torch.uint8, device=DEV)
        B.grem_set_workspace(ws)
        try:
            sd_d = torch.as_tensor(seed).to(DEV)
            out = B.grem_partition_planned(plan, 3, 1.05, 2, sd_d, want_sizes=True, want_estimates=False)
            torch.cuda.synchronize()
            assert np.array_equal(out[0].cpu().numpy(), oracle.partition_seeded(g.rowptr, g.colidx, g.n, 3, 1.05, chunk, 2, seed))
            B.grem_set_workspace(ws[:1 << 16])
            with pytest.raises(B.GremError) as e:
                B.grem_partition_planned(plan, 16, 1.05, 2)
            assert e.value.code == B.ERR_NOMEM
        finally:
            B.grem_set_workspace(None)
        del ci                                  # the plan does not read colidx after it has been built
        torch.cuda.empty_cache()
        for k, slack, R, sd in ((16, 1.05, 2, None), (3, 1.0, 1, seed), (16, 1.05, 2, None), (7, 1.3, 0, None),
                                (1, 1.0, 1, None), (13, 1.02, 6, None), (5, 1.1, 9, seed)):
            print(f"[case] planned run k={k} slack={slack} R={R} seeded={sd is not None}", flush=True)
            sd_d = None if sd is None else torch.as_tensor(sd).to(DEV)
            out = B.grem_partition_planned(plan, k, slack, R, sd_d, want_sizes=True, want_estimates=True)
            torch.cuda.synchronize()
            _same_as_oracle(g, out, k, slack, chunk, R, sd)
            # labels only (the last pass then does not store the estimates)
            lab = B.grem_partition_planned(plan, k, slack, R, sd_d)
            torch.cuda.synchronize()
            assert torch.equal(lab, out[0])


def test_a_plan_for_up_to_32_partitions():
    g, rp, ci = _dev(synth.hub_stress(scale=14, edge_factor=8, hubs=3, hub_degree=3000, seed=2))
    chunk = 3000
    with B.Plan(rp, ci, g.n, chunk, B.options(col_bits=9, hub_degree=300, plan_max_k=32)) as plan:
        assert plan.max_k == 32
        for k, slack, R in ((32, 1.05, 2), (8, 1.05, 1), (21, 1.0, 2), (16, 1.1, 0)):
            print(f"[case] planned run on a plan for 32: k={k} slack={slack} R={R}", flush=True)
            out = B.grem_partition_planned(plan, k, slack, R, want_sizes=True, want_estimates=True)
            torch.cuda.synchronize()
            _same_as_oracle(g, out, k, slack, chunk, R)
    with B.Plan(rp, ci, g.n, chunk, B.options(col_bits=9, hub_degree=300)) as plan:
        assert plan.max_k == 16
        with pytest.raises(B.GremError) as e:
            B.grem_partition_planned(plan, 17, 1.05, 1)
        assert e.value.code == B.ERR_ARG


def test_planned_run_equals_the_unplanned_call():
    g, rp, ci = _dev(synth.chung_lu(300_000, 3_000_000, gamma=2.1, cap=5_000.0, seed=4))
    chunk, k = 1 << 15, 16
    want = B.grem_partition(rp, ci, g.n, k, 1.05, chunk, 2, options=B.options(B.HIST_LDS))
    with B.Plan(rp, ci, g.n, chunk) as plan:
        got = B.grem_partition_planned(plan, k, 1.05, 2)
        torch.cuda.synchronize()
    assert torch.equal(got, want)
    assert np.array_equal(got.cpu().numpy(), oracle.partition(g.rowptr, g.colidx, g.n, k, 1.05, chunk, 2))


def test_plan_errors():
    g, rp, ci = _dev(synth.random_graph_np(500, 3000, 1))
    with pytest.raises(B.GremError) as e:
        B.Plan(rp, ci, g.n, 0)
    assert e.value.code == B.ERR_ARG
    with pytest.raises(B.GremError) as e:
        B.Plan(rp, ci, g.n, 100, B.options(col_bits=2))
    assert e.value.code == B.ERR_ARG
    with B.Plan(rp, ci, g.n, 100, B.options(col_bits=5, hub_degree=8)) as plan:
        for bad in (dict(k=0), dict(k=17), dict(R=-1), dict(slack=0.5)):
            a = dict(k=4, R=1, slack=1.05)
            a.update(bad)
            with pytest.raises(B.GremError) as e:
                B.grem_partition_planned(plan, a["k"], a["slack"], a["R"])
            assert e.value.code == B.ERR_ARG
        with pytest.raises(B.GremError) as e:
            B.grem_partition_planned(plan, 4, 1.05, 31)
        assert e.value.code == B.ERR_RANGE
        seed = torch.full((g.n,), 7, dtype=torch.int32, device=DEV)
        with pytest.raises(B.GremError) as e:
            B.grem_partition_planned(plan, 4, 1.05, 1, seed)
        assert e.value.code == B.ERR_SEED
        lab = B.grem_partition_planned(plan, 4, 1.05, 1)
        torch.cuda.synchronize()
        assert lab.cpu().numpy().tolist() == oracle.partition(g.rowptr, g.colidx, g.n, 4, 1.05, 100, 1).tolist()


def test_concurrent_calls_on_two_streams():
    # two different runs enqueued back to back on two streams (each call keeps its state in memory of its own),
    # then two runs on one plan at once; all four equal the oracle
    ga, rpa, cia = _dev(synth.rmat(17, 16, seed=3))
    gb, rpb, cib = _dev(synth.chung_lu(200_000, 2_000_000, gamma=2.1, cap=2_000.0, seed=9))
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for round_ in range(3):
        with torch.cuda.stream(s1):
            outa = B.grem_partition_state(rpa, cia, ga.n, 8, 1.05, 1 << 13, 2, stream=s1,
                                          options=B.options(B.HIST_SWEEP, col_bits=11, hub_degree=500))
        with torch.cuda.stream(s2):
            outb = B.grem_partition_state(rpb, cib, gb.n, 48, 1.1, 20_000, 1, stream=s2)
        s1.synchronize()
        s2.synchronize()
        if round_ == 0:
            _same_as_oracle(ga, outa, 8, 1.05, 1 << 13, 2)
            _same_as_oracle(gb, outb, 48, 1.1, 20_000, 1)
            first = (outa[0].clone(), outb[0].clone())
        else:
            assert torch.equal(outa[0], first[0]) and torch.equal(outb[0], first[1])
    with B.Plan(rpa, cia, ga.n, 1 << 13, B.options(col_bits=11, hub_degree=500)) as plan:
        with torch.cuda.stream(s1):
            o1 = B.grem_partition_planned(plan, 8, 1.05, 2, want_sizes=True, want_estimates=True, stream=s1)
        with torch.cuda.stream(s2):
            o2 = B.grem_partition_planned(plan, 5, 1.2, 3, want_sizes=True, want_estimates=True, stream=s2)
        s1.synchronize()
        s2.synchronize()
        _same_as_oracle(ga, o1, 8, 1.05, 1 << 13, 2)
        _same_as_oracle(ga, o2, 5, 1.2, 1 << 13, 3)
