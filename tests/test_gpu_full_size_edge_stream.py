"""Full-size checks of the edge-chunk path on the stream of the bench workload (Chung-Lu graph with
111M nodes, 1.6e9 undirected edges in random order, chunks of 1 % of the edges, two partitions):
  * the run over the first three chunks alone equals the oracle's element by element (parts, sizes,
    estimates as raw doubles);
  * a longer prefix whose first chunk is seeded entirely with partition 0, so that partition 0 reaches its
    capacity inside the prefix (requests rejected by rank, new nodes placed in the other partition, and
    later chunks deciding against a full partition), equals the oracle's in the same way;
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


def test_prefix_that_fills_a_partition_equals_the_oracle(stream):
    es, _, c_size, P = stream
    seed0 = np.zeros(es.n, dtype=np.int32)        # every first-chunk node starts in partition 0
    # partition 0 then grows fastest and runs out of room after about ten chunks.  The oracle is stepped until
    # two chunks after the first one in which requests were turned down (a node's request differs from the
    # partition it ends the chunk in: refused by rank, and placed in the other partition if it was new).
    limit = 20
    m = limit * c_size
    src_h, dst_h = es.src[:m].cpu().numpy(), es.dst[:m].cpu().numpy()
    st = oracle.EdgeStepper(src_h, dst_h, es.n, c_size, P, seed0)
    chunks, first_refusal, refused = 0, None, 0
    while chunks < limit and (first_refusal is None or chunks < first_refusal + 3):
        assert st.step()
        chunks += 1
        nodes, _, prop = st.last_chunk()
        if chunks > 1:
            after = st.parts()[nodes]
            turned_down = int(((prop >= 0) & (prop != after)).sum())
            print(f"[oracle] chunk {chunks}: {nodes.size} nodes, {turned_down} requests turned down, sizes "
                  f"{st.sizes().tolist()}", flush=True)
            if turned_down and first_refusal is None:
                first_refusal = chunks
            refused += turned_down
    assert first_refusal is not None, f"no request was turned down within {limit} chunks"
    oparts, osizes, oest = st.parts(), st.sizes(), st.nbr_counts()
    st.close()
    m = chunks * c_size
    print(f"[case] edge stream prefix parity with a full partition: {chunks} chunks of {c_size} edges, "
          f"{refused} requests turned down", flush=True)
    src, dst = es.src[:m].contiguous(), es.dst[:m].contiguous()
    parts, sizes, est = B.grem_edge_stream_bipartition(src, dst, es.n, c_size, P, torch.as_tensor(seed0).to(DEV))
    torch.cuda.synchronize()
    assert np.array_equal(parts.cpu().numpy(), oparts)
    assert sizes.cpu().numpy().tolist() == osizes.tolist()
    assert np.array_equal(est.cpu().numpy().view(np.uint64), oest.view(np.uint64))


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


def test_recursive_bisection_full_size_properties(stream):
    # 16 partitions of the same stream by four levels of bisection: label range, the compound capacity
    # bound, the levels' prefix property (a shallower run equals the deeper run's leading bits), and the
    # first level equal to the two-partition entry point followed by the placement of untouched nodes
    es, _, _, _ = stream
    n, levels, chunks, slack = es.n, 4, 100, 1.05 ** 0.25
    ids = torch.arange(n, device=DEV, dtype=torch.int32)
    bits = torch.stack([(ids >> l) & 1 for l in range(levels)]).contiguous()
    print("[case] recursive bisection, 4 levels, full size", flush=True)
    lab4 = B.grem_recursive_bisection(es.src, es.dst, n, levels, chunks, slack, bits.reshape(-1))
    torch.cuda.synchronize()
    assert int(lab4.min()) >= 0 and int(lab4.max()) < 16
    sizes = torch.bincount(lab4, minlength=16)
    cap = n
    for _ in range(levels):
        cap = B.grem_capacity(cap, 2, slack)
    assert int(sizes.sum()) == n and int(sizes.max()) <= cap
    print("[case] recursive bisection, 1 level, full size", flush=True)
    lab1 = B.grem_recursive_bisection(es.src, es.dst, n, 1, chunks, slack, bits[0].contiguous())
    torch.cuda.synchronize()
    assert torch.equal(lab1, lab4 >> 3)
    c_size = (es.m + chunks - 1) // chunks
    P = B.grem_capacity(n, 2, slack)
    parts, psizes, _ = B.grem_edge_stream_bipartition(es.src, es.dst, n, c_size, P, bits[0].contiguous(),
                                                      want_nbr_counts=False)
    torch.cuda.synchronize()
    touched = parts >= 0
    assert torch.equal(lab1[touched], parts[touched])
    # untouched nodes, ascending id: the first |S0 - S1| go to the smaller half, the rest alternate 0,1,...
    a, b = int(psizes[0]), int(psizes[1])
    free = torch.nonzero(~touched).flatten()
    j = torch.arange(free.numel(), device=DEV)
    gap = abs(a - b)
    want = torch.where(j < gap, torch.full_like(j, 0 if a <= b else 1), (j - gap) & 1).to(torch.int32)
    assert torch.equal(lab1[free], want)
    cut = int(B.grem_edge_list_cut(es.src, es.dst, lab4).item())
    print(f"[result] 16-way cut fraction by recursive bisection {cut / es.m:.4f}", flush=True)
    assert cut < (15 / 16) * es.m
