"""Full-size checks of the edge-chunk path on the stream of the bench workload (Chung-Lu graph with
111M nodes, 1.6e9 undirected edges in random order, chunks of 1 % of the edges, two partitions):
  * the run over the first three chunks alone equals the oracle's element by element (parts, sizes,
    estimates as raw doubles);
  * the whole run is checked through properties that hold at any size, is repeatable bit for bit,
    and refined decisions cut fewer edges than fixed greedy ones (Sec. 4.2, Fig. 7)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2502_17846_amd import binding as B
from paper_2502_17846_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
N, M, FRAC, SLACK = 111_000_000, 1_600_000_000, 0.01, 1.05


@pytest.fixture(scope="module")
def stream():
    g = synth.chung_lu(N, M, gamma=2.1, cap=50_000.0, seed=0, device=DEV, rowptr_dtype=torch.int64)
    es = synth.edge_stream(g, seed=1)
    del g
    torch.cuda.empty_cache()
    seed = (torch.arange(es.n, device=DEV, dtype=torch.int32) & 1)
    return es, seed, max(1, int(round(es.m * FRAC))), B.grem_capacity(es.n, 2, SLACK)


def test_first_chunks_equal_the_oracle(stream):
    es, seed, c_size, P = stream
    chunks = 3
    m = chunks * c_size
    print(f"[case] edge stream prefix parity: {chunks} chunks of {c_size} edges, n={es.n}", flush=True)
    src, dst = es.src[:m].contiguous(), es.dst[:m].contiguous()
    parts, sizes, est = B.grem_edge_stream_bipartition(src, dst, es.n, c_size, P, seed)
    torch.cuda.synchronize()
    oparts, osizes, oest = oracle.edge_stream_bipartition(src.cpu().numpy(), dst.cpu().numpy(), es.n, c_size, P,
                                                          seed.cpu().numpy(), return_state=True)
    assert np.array_equal(parts.cpu().numpy(), oparts)
    assert sizes.cpu().numpy().tolist() == osizes.tolist()
    assert np.array_equal(est.cpu().numpy().view(np.uint64), oest.view(np.uint64))
    assert int((oparts >= 0).sum()) > 30_000_000          # the prefix does reach a large part of the graph


def test_whole_run_properties(stream):
    es, seed, c_size, P = stream
    touched = torch.zeros(es.n, dtype=torch.bool, device=DEV)
    touched[es.src.long()] = True
    touched[es.dst.long()] = True
    cuts = {}
    for mode in (B.EDGE_REFINE, B.EDGE_FIXED):
        print(f"[case] edge stream whole run, mode {mode}", flush=True)
        parts, sizes, est = B.grem_edge_stream_bipartition(es.src, es.dst, es.n, c_size, P, seed, mode)
        cut = B.grem_edge_list_cut(es.src, es.dst, parts)
        torch.cuda.synchronize()
        assert torch.equal(parts >= 0, touched)
        assert int(parts.max()) <= 1 and int(parts.min()) >= -1
        cnt = torch.bincount(parts[touched], minlength=2)
        assert torch.equal(cnt, sizes) and int(cnt.max()) <= P
        assert bool((est[~touched] == 0).all()) and bool((est >= 0).all())
        assert int(cut.item()) == int((parts[es.src.long()] != parts[es.dst.long()]).sum().item())
        cuts[mode] = int(cut.item())
        if mode == B.EDGE_REFINE:
            parts2, sizes2, est2 = B.grem_edge_stream_bipartition(es.src, es.dst, es.n, c_size, P, seed, mode)
            torch.cuda.synchronize()
            assert torch.equal(parts, parts2) and torch.equal(sizes, sizes2)
            assert torch.equal(est.view(torch.int64), est2.view(torch.int64))
            del parts2, sizes2, est2
        del parts, sizes, est
    print(f"[result] cut fraction refined {cuts[B.EDGE_REFINE] / es.m:.4f}, fixed {cuts[B.EDGE_FIXED] / es.m:.4f}", flush=True)
    assert cuts[B.EDGE_REFINE] < cuts[B.EDGE_FIXED]
    assert cuts[B.EDGE_REFINE] < 0.5 * es.m               # better than a random bisection
