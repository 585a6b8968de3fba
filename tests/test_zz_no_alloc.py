"""The entry point that allocates nothing (grem_expected_cut_noalloc: for callers that cannot call
hipMalloc) against grem_expected_cut, through the C ABI: two calls in a row, the second on a smaller input,
so that whatever the first call left in the library's fixed buffer must not leak into the second."""
import numpy as np
import pytest
import torch

from paper_2502_17846_amd import binding as B
from paper_2502_17846_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
RTOL = 1e-9       # the bar of the Eq. (1) parity tests; the two entry points share their kernels and the order
                  # of every sum, so the outputs are in fact compared bit for bit as well


def _t(a, dtype=None):
    t = torch.as_tensor(np.ascontiguousarray(a))
    return t.to(device=DEV) if dtype is None else t.to(device=DEV, dtype=dtype)


def _case(g, x, rdt):
    labels = np.random.default_rng(11).integers(-1, 2, g.n).astype(np.int32)
    return _t(g.rowptr, rdt), _t(g.colidx), g.n, _t(labels), x


def test_two_calls_in_a_row_equal_the_allocating_entry_point():
    big = synth.to_numpy(synth.rmat(16, 16, seed=5))                    # 65,536 rows: 4,096 workgroups
    small = synth.planted_partition(n=3_000, blocks=2, mean_degree=9.0, seed=6)   # 188 workgroups, ragged tail
    out = torch.full((2,), float("nan"), dtype=torch.float64, device=DEV)
    for g, x, rdt in ((big, 0.05, torch.int64), (small, 0.3, torch.int32)):
        rp, ci, n, lab, x = _case(g, x, rdt)
        want = B.grem_expected_cut(rp, ci, n, lab, x)
        torch.cuda.synchronize()
        out.fill_(float("nan"))
        got = B.grem_expected_cut_noalloc(rp, ci, n, lab, x, out)
        torch.cuda.synchronize()
        w, g_ = want.cpu().numpy(), got.cpu().numpy()
        print(f"[case] n={n} x={x}: {g_.tolist()} vs {w.tolist()}", flush=True)
        assert np.all(np.isfinite(g_))
        assert g_[1] == w[1]
        assert abs(g_[0] - w[0]) <= RTOL * max(1.0, abs(w[0]))
        assert np.array_equal(g_.view(np.uint64), w.view(np.uint64))


def test_sizes_beyond_the_buffer_are_refused():
    limit = B.grem_expected_cut_noalloc_max_n()
    assert limit == 4_194_304
    n = limit + 1
    rp = torch.zeros(n + 1, dtype=torch.int32, device=DEV)
    ci = torch.zeros(1, dtype=torch.int32, device=DEV)
    lab = torch.zeros(n, dtype=torch.int32, device=DEV)
    out = torch.zeros(2, dtype=torch.float64, device=DEV)
    with pytest.raises(B.GremError) as e:
        B.grem_expected_cut_noalloc(rp, ci, n, lab, 0.5, out)
    assert e.value.code == B.ERR_LIMIT
    # at the limit itself (an edgeless graph: every term is zero) the call goes through
    got = B.grem_expected_cut_noalloc(rp[:limit + 1], ci, limit, lab[:limit], 0.5, out)
    torch.cuda.synchronize()
    assert got.cpu().numpy().tolist() == [0.0, 0.0]
