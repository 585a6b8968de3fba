"""Full-size checks of the R-MAT scale 27 workload (134M vertices, 8.4e9 CSR entries, int64 rowptr,
k=32, slack 1.03, chunk 2^22, 1 refinement pass): the largest graph of the set, more than 2^32 entries.
  * refine_passes = 0: labels and estimates of the first chunks are final after pass 0 and depend only on
    those chunks' rows; they are compared element by element with the oracle stepped over the same prefix,
    which is long enough that its last chunk's entries lie beyond offset 2^32 of colidx, holds rows of
    16,384 entries and more, and (from the second chunk on) counts labelled neighbours;
  * the 2-pass run is checked through properties that hold at any size, and two routes must agree bit
    for bit: LDS histograms with long rows split off, and histograms in E's rows with nothing split off."""
import numpy as np
import pytest
import torch

import oracle
from paper_2502_17846_amd import binding as B
from paper_2502_17846_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
K, SLACK, CHUNK, R = 32, 1.03, 1 << 22, 1


@pytest.fixture(scope="module")
def graph():
    g = synth.rmat(27, 32, seed=0, device=DEV, rowptr_dtype=torch.int64)
    ws = torch.empty(B.grem_workspace_bytes_two_phase(g.n, g.nnz, K, CHUNK), dtype=torch.uint8, device=DEV)
    B.grem_set_workspace(ws)
    yield g
    B.grem_set_workspace(None)


def test_first_chunks_of_pass0_equal_the_oracle(graph):
    g = graph
    assert g.nnz > 2**32
    # the shortest prefix of whole chunks whose last chunk starts beyond entry 2^32
    nchunks = (g.n + CHUNK - 1) // CHUNK
    starts = g.rowptr[torch.arange(nchunks, device=DEV) * CHUNK]
    chunks = int((starts <= 2**32).sum().item()) + 1
    assert 2 <= chunks <= nchunks and int(starts[chunks - 1].item()) > 2**32
    rows = chunks * CHUNK
    end = int(g.rowptr[rows].item())
    deg = g.rowptr[1:rows + 1] - g.rowptr[:rows]
    print(f"[case] rmat-27 prefix parity, {chunks} chunks, {end} entries, rows of >= 16384 entries in it: "
          f"{int((deg >= 16384).sum())}", flush=True)
    assert int((deg >= 16384).sum()) > 0
    del deg
    rp = g.rowptr.cpu().numpy().copy()
    rp[rows:] = end
    ci = g.colidx[:end].cpu().numpy()
    st = oracle.Stepper(rp, ci, g.n, K, SLACK, CHUNK, 0)
    for c in range(chunks):
        st.step()
        print(f"[oracle] chunk {c + 1} of {chunks}", flush=True)
    olab, oest = st.labels()[:rows].copy(), st.estimates()[:rows].copy()
    st.close()
    del rp, ci
    assert oest[CHUNK:].any() and oest[(chunks - 1) * CHUNK:].any()     # labelled neighbours were counted
    lab, sizes, est = B.grem_partition_state(g.rowptr, g.colidx, g.n, K, SLACK, CHUNK, 0)
    torch.cuda.synchronize()
    assert np.array_equal(lab[:rows].cpu().numpy(), olab)
    assert np.array_equal(est[:rows].cpu().numpy().view(np.uint32), oest)


def test_two_pass_run_properties_and_route_agreement(graph):
    g = graph
    P = B.grem_capacity(g.n, K, SLACK)
    assert P == oracle.capacity(g.n, K, SLACK) == 4_320_134
    outs = []
    for mode, long_deg, what in ((B.HIST_AUTO, 0, "LDS histograms, long rows split off"),
                                 (B.HIST_GLOBAL, 2**31 - 1, "histograms in E's rows, nothing split off")):
        print(f"[case] rmat-27 2-pass run: {what}", flush=True)
        lab, sizes, _ = B.grem_partition_state(g.rowptr, g.colidx, g.n, K, SLACK, CHUNK, R, want_estimates=False,
                                               options=B.options(mode, long_row_degree=long_deg))
        cut = B.grem_edge_cut(g.rowptr, g.colidx, g.n, lab)
        torch.cuda.synchronize()
        assert int(lab.min()) >= 0 and int(lab.max()) < K
        cnt = torch.bincount(lab, minlength=K)
        assert torch.equal(cnt, sizes) and int(cnt.max()) <= P and int(cnt.sum()) == g.n
        outs.append((lab, int(cut.item())))
    assert torch.equal(outs[0][0], outs[1][0])
    assert outs[0][1] == outs[1][1]
    assert outs[0][1] / g.nnz < 31 / 32         # better than a random 32-way split
