"""Full-size checks of the bench workload (111M vertices, 3.19e9 CSR entries, k=16, chunk 2^20) in the
launch configuration bench.py times:
  * with refine_passes = 0 the labels of the first chunks are final after pass 0 and depend only on those
    chunks' rows: they are compared, element by element, with the oracle stepped over the same prefix
    (unseeded and seeded);
  * the whole 3-pass run is checked through properties that hold at any size (label range, sizes equal
    the label counts and respect the capacity, two runs give the same bytes) and the two independent
    score paths (plain LDS and two-phase) must agree bit for bit;
  * a labelling evaluated on a plan (neighbour counts, cut, Eq. (1)): sampled rows of the counts equal the
    oracle's, the cut equals the walk over the CSR arrays, Eq. (1) agrees with the CSR routine;
  * the complete 3-pass run (pass 0 and two refinement passes, 318 chunk steps) is replayed on the oracle
    (two to three minutes of single-thread CPU time) and labels, sizes and estimates are compared element
    by element with the library's."""
import numpy as np
import pytest
import torch

import oracle
from paper_2502_17846_amd import binding as B
from paper_2502_17846_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
N, M, K, SLACK, CHUNK = 111_000_000, 1_600_000_000, 16, 1.05, 1 << 20


@pytest.fixture(scope="module")
def graph():
    g = synth.chung_lu(N, M, gamma=2.1, cap=50_000.0, seed=0, device=DEV, rowptr_dtype=torch.int64)
    ws = torch.empty(B.grem_workspace_bytes_two_phase(g.n, g.nnz, K, CHUNK), dtype=torch.uint8, device=DEV)
    B.grem_set_workspace(ws)
    yield g
    B.grem_set_workspace(None)


def _prefix_oracle(g, chunks):
    rows = chunks * CHUNK
    end = int(g.rowptr[rows].item())
    rp = g.rowptr.cpu().numpy().copy()
    rp[rows:] = end
    ci = g.colidx[:end].cpu().numpy()
    st = oracle.Stepper(rp, ci, g.n, K, SLACK, CHUNK, 0)
    for _ in range(chunks):
        st.step()
    lab, est = st.labels()[:rows], st.estimates()[:rows]
    st.close()
    return lab, est


def test_first_chunks_of_pass0_equal_the_oracle(graph):
    g = graph
    chunks = 3
    print(f"[case] full-size prefix parity, {chunks} chunks", flush=True)
    olab, oest = _prefix_oracle(g, chunks)
    rows = chunks * CHUNK
    for mode in (B.HIST_AUTO, B.HIST_LDS):
        lab, sizes, est = B.grem_partition_state(g.rowptr, g.colidx, g.n, K, SLACK, CHUNK, 0, options=B.options(mode))
        torch.cuda.synchronize()
        assert np.array_equal(lab[:rows].cpu().numpy(), olab), f"mode {mode}"
        assert np.array_equal(est[:rows].cpu().numpy().view(np.uint32), oest), f"mode {mode}"
        del lab, sizes, est


def test_seeded_first_chunks_of_pass0_equal_the_oracle(graph):
    # a tenth of all vertices start with a (random) label: in the first pass their rows keep it, and every
    # other row counts them wherever they lie, while the rest of its neighbours further on are unassigned
    g = graph
    chunks = 2
    rows = chunks * CHUNK
    rng = np.random.default_rng(7)
    seed = np.where(rng.random(g.n) < 0.1, rng.integers(0, K, g.n), -1).astype(np.int32)
    print(f"[case] full-size seeded prefix parity, {chunks} chunks, {(seed >= 0).sum()} seeds", flush=True)
    end = int(g.rowptr[rows].item())
    rp = g.rowptr.cpu().numpy().copy()
    rp[rows:] = end
    ci = g.colidx[:end].cpu().numpy()
    st = oracle.Stepper(rp, ci, g.n, K, SLACK, CHUNK, 0, seed_labels=seed)
    for _ in range(chunks):
        st.step()
    olab, oest = st.labels()[:rows].copy(), st.estimates()[:rows].copy()
    st.close()
    seed_d = torch.as_tensor(seed).to(DEV)
    lab, sizes, est = B.grem_partition_state(g.rowptr, g.colidx, g.n, K, SLACK, CHUNK, 0, seed_d)
    torch.cuda.synchronize()
    assert np.array_equal(lab[:rows].cpu().numpy(), olab)
    assert np.array_equal(est[:rows].cpu().numpy().view(np.uint32), oest)
    keep = torch.as_tensor(seed >= 0).to(DEV)
    assert torch.equal(lab[keep], seed_d[keep])         # a seeded vertex keeps its seed in the first pass
    del lab, sizes, est
    # one refinement pass on top: the two-phase path and the plain path agree on the whole seeded run
    outs = []
    for mode in (B.HIST_AUTO, B.HIST_LDS):
        lab, sizes, _ = B.grem_partition_state(g.rowptr, g.colidx, g.n, K, SLACK, CHUNK, 1, seed_d,
                                               want_estimates=False, options=B.options(mode))
        torch.cuda.synchronize()
        assert torch.equal(torch.bincount(lab, minlength=K), sizes)
        outs.append(lab)
    assert torch.equal(outs[0], outs[1])


def test_three_pass_run_properties_and_path_agreement(graph):
    g = graph
    P = B.grem_capacity(g.n, K, SLACK)
    assert P == oracle.capacity(g.n, K, SLACK) == 7_284_375
    outs = []
    for mode in (B.HIST_AUTO, B.HIST_AUTO, B.HIST_LDS):
        print(f"[case] full-size 3-pass run, mode {mode}", flush=True)
        lab, sizes, _ = B.grem_partition_state(g.rowptr, g.colidx, g.n, K, SLACK, CHUNK, 2,
                                               want_estimates=False, options=B.options(mode))
        cut = B.grem_edge_cut(g.rowptr, g.colidx, g.n, lab)
        torch.cuda.synchronize()
        assert int(lab.min()) >= 0 and int(lab.max()) < K
        cnt = torch.bincount(lab, minlength=K)
        assert torch.equal(cnt, sizes) and int(cnt.max()) <= P and int(cnt.sum()) == g.n
        outs.append((lab, int(cut.item())))
    assert torch.equal(outs[0][0], outs[1][0])          # same bytes on repeat
    assert torch.equal(outs[0][0], outs[2][0])          # column-sliced path == plain path
    assert outs[0][1] == outs[2][1]
    # the cut of a random 16-way split is 15/16; the run must do better than that
    assert outs[0][1] / g.nnz < 15 / 16


def test_a_labelling_evaluated_on_a_plan(graph):
    g = graph
    print("[case] full-size plan: neighbour counts, cut, Eq. (1)", flush=True)
    with B.Plan(g.rowptr, g.colidx, g.n, CHUNK) as plan:
        lab = B.grem_partition_planned(plan, K, SLACK, 0)
        lab[::1000] = -1                                   # some vertices without a label
        counts = B.grem_plan_neighbour_counts(plan, K, lab)
        cut = B.grem_plan_edge_cut(plan, K, lab)
        torch.cuda.synchronize()
        assert int(cut.item()) == int(B.grem_edge_cut(g.rowptr, g.colidx, g.n, lab).item())
        # rows sampled over the whole range (hubs among them: the 2,000 longest rows), against the oracle
        rng = np.random.default_rng(3)
        deg = g.rowptr[1:] - g.rowptr[:-1]
        rows = torch.cat([torch.as_tensor(rng.integers(0, g.n, 20_000)).to(DEV), torch.topk(deg, 2000).indices,
                          torch.arange(g.n - 64, g.n, device=DEV)]).unique()
        lens = deg[rows]
        sub_rp = torch.zeros(rows.numel() + 1, dtype=torch.int64, device=DEV)
        sub_rp[1:] = torch.cumsum(lens, 0)
        pos = torch.arange(int(sub_rp[-1].item()), device=DEV) - torch.repeat_interleave(sub_rp[:-1] - g.rowptr[rows], lens)
        sub_ci = g.colidx[pos]
        want = oracle.neighbour_counts(sub_rp.cpu().numpy(), sub_ci.cpu().numpy(), rows.numel(), lab.cpu().numpy(), K)
        got = counts[rows].cpu().numpy().view(np.uint32).astype(np.int64)
        assert int(lens.max()) > 40_000 and np.array_equal(got, want)
        del counts, pos, sub_ci
        two = torch.where(lab >= 0, lab & 1, lab)
        a = B.grem_plan_expected_cut(plan, two, 0.01)
        b = B.grem_expected_cut(g.rowptr, g.colidx, g.n, two, 0.01)
        torch.cuda.synchronize()
        a, b = a.cpu().numpy(), b.cpu().numpy()
        assert a[1] == b[1] and abs(a[0] - b[0]) <= 1e-9 * b[0]


def test_whole_run_equals_the_oracle(graph):
    g = graph
    rp, ci = g.rowptr.cpu().numpy(), g.colidx.cpu().numpy()
    print("[case] full-size whole-run oracle replay", flush=True)
    st = oracle.Stepper(rp, ci, g.n, K, SLACK, CHUNK, 2)
    steps = 0
    while st.step():
        steps += 1
        if steps % 20 == 0:
            print(f"[oracle] {steps} chunk steps", flush=True)
    assert steps == 3 * ((g.n + CHUNK - 1) // CHUNK)
    olab, osizes, oest = st.labels(), st.sizes(), st.estimates()
    st.close()
    del rp, ci
    # the call bench.py times (labels only: the last pass does not store the estimates) ...
    lab = B.grem_partition(g.rowptr, g.colidx, g.n, K, SLACK, CHUNK, 2)
    torch.cuda.synchronize()
    assert np.array_equal(lab.cpu().numpy(), olab)
    del lab
    # ... and the same run returning all of Alg. 1's state
    lab, sizes, est = B.grem_partition_state(g.rowptr, g.colidx, g.n, K, SLACK, CHUNK, 2)
    torch.cuda.synchronize()
    assert np.array_equal(lab.cpu().numpy(), olab)
    assert sizes.cpu().numpy().tolist() == osizes.tolist()
    assert np.array_equal(est.cpu().numpy().view(np.uint32), oest)
