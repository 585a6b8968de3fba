"""CPU pins of the edge-chunk oracle (Alg. 1 in the paper's own stream model, two partitions).

Each test states which mistake it is meant to catch."""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2502_17846_amd import synth
from tests import ref_models as ref

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _run(src, dst, n, c_size, P, seed, mode=oracle.EDGE_REFINE):
    return oracle.edge_stream_bipartition(src, dst, n, c_size, P, seed, mode, return_state=True)


# ---------------------------------------------------------------------------------------------
# hand-worked examples: the whole rule on inputs small enough to follow on paper (wrong tie
# direction, missing removal before assign, rank test off by one, spill target, blend weights,
# loops, unassigned neighbours, the fixed-greedy switch)
# ---------------------------------------------------------------------------------------------

def test_handworked_examples():
    with open(os.path.join(GOLDEN, "handworked_edge_stream.json")) as f:
        cases = json.load(f)["cases"]
    for c in cases:
        e = np.asarray(c["edges"], dtype=np.int32)
        seed = np.asarray(c["seed_parts"], dtype=np.int32)
        for key, mode in (("refine", oracle.EDGE_REFINE), ("fixed", oracle.EDGE_FIXED)):
            if key not in c:
                continue
            parts, sizes, est = _run(e[:, 0], e[:, 1], c["n"], c["c_size"], c["P"], seed, mode)
            want = c[key]
            assert parts.tolist() == want["parts"], (c["name"], key)
            assert sizes.tolist() == want["sizes"], (c["name"], key)
            assert est.tolist() == want["nbr_counts"], (c["name"], key)
            assert oracle.edge_list_cut(e[:, 0], e[:, 1], parts) == want["cut"], (c["name"], key)


# ---------------------------------------------------------------------------------------------
# the literal node-at-a-time procedure, wherever it detects no dependence inside a chunk
# ---------------------------------------------------------------------------------------------

def _growing_stream(rng, n, m, p_new):
    """Edges whose new endpoint (if any) has the next unused id, so that a new node's chunk
    neighbours have lower ids and are evaluated before it; the first two nodes start the stream."""
    src, dst = [0], [1]
    used = 2
    while len(src) < m:
        if used < n and rng.random() < p_new:
            a, b = int(rng.integers(0, used)), used
            used += 1
        else:
            a, b = int(rng.integers(0, used)), int(rng.integers(0, used))
        if rng.random() < 0.5:
            a, b = b, a
        src.append(a)
        dst.append(b)
    return np.asarray(src, np.int32), np.asarray(dst, np.int32), used


@pytest.mark.parametrize("refine", [True, False])
def test_equals_sequential_procedure_when_chunks_have_no_inner_dependence(refine):
    rng = np.random.default_rng(5 if refine else 6)
    compared = tight = 0
    for trial in range(1500):
        n = int(rng.integers(4, 14))
        m = int(rng.integers(3, 30))
        c_size = int(rng.integers(1, 5))
        src, dst, used = _growing_stream(rng, n, m, float(rng.uniform(0.2, 0.7)))
        P = int(rng.integers((n + 1) // 2, n + 1))
        seed = rng.integers(0, 2, n).astype(np.int32)
        first = np.unique(np.concatenate([src[:c_size], dst[:c_size]]))
        if max(np.sum(seed[first] == 0), np.sum(seed[first] == 1)) > P:
            continue
        sp, ss, se, dependent = ref.sequential_edge_stream(src, dst, n, c_size, P, seed, refine)
        if dependent:
            continue
        parts, sizes, est = _run(src, dst, n, c_size, P, seed,
                                 oracle.EDGE_REFINE if refine else oracle.EDGE_FIXED)
        assert parts.tolist() == sp, (trial, src.tolist(), dst.tolist(), c_size, P, seed.tolist())
        assert sizes.tolist() == ss
        assert [[Fraction(x) for x in row] for row in est.tolist()] == se
        compared += 1
        tight += int(max(ss) == P)
    assert compared >= 100 and tight >= 10, (compared, tight)


# ---------------------------------------------------------------------------------------------
# counts and chunk nodes against dense incidence algebra; invariants after every chunk; the
# closed-form chunk weights of Sec. 4.1 (first two appearances equal, then halving)
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("seed_,loops", [(0, False), (1, True), (2, True)])
def test_counts_weights_and_invariants_chunk_by_chunk(seed_, loops):
    rng = np.random.default_rng(seed_)
    n, m, c_size = 40, 300, 17
    src = rng.integers(0, n - 3, m).astype(np.int32)       # the last 3 nodes never occur
    dst = rng.integers(0, n - 3, m).astype(np.int32)
    if not loops:
        dst = np.where(dst == src, (dst + 1) % (n - 3), dst).astype(np.int32)
    P = 21
    seed = rng.integers(0, 2, n).astype(np.int32)
    st = oracle.EdgeStepper(src, dst, n, c_size, P, seed)
    history = [[] for _ in range(n)]           # per node: fresh counts of every chunk it occurred in
    prev = st.parts()
    chunk = 0
    while True:
        before = prev.copy()
        if not st.step():
            break
        lo, hi = chunk * c_size, min(m, (chunk + 1) * c_size)
        nodes, fresh, prop = st.last_chunk()
        assert nodes.tolist() == np.unique(np.concatenate([src[lo:hi], dst[lo:hi]])).tolist()
        if chunk == 0:
            before[nodes] = seed[nodes]
        M = ref.chunk_incidence(src[lo:hi], dst[lo:hi], n)
        onehot = np.stack([(before == 0), (before == 1)], axis=1).astype(np.int64)
        assert np.array_equal(fresh, (M @ onehot)[nodes])
        now, sizes = st.parts(), st.sizes()
        assert sizes.tolist() == [int((now == 0).sum()), int((now == 1).sum())]
        assert sizes.max() <= P
        changed = np.nonzero(now != before)[0]
        assert set(changed.tolist()) <= set(nodes.tolist())
        assert np.all(now[nodes] >= 0)
        for v, f in zip(nodes.tolist(), fresh.tolist()):
            history[v].append(f)
        est = st.nbr_counts()
        for v in nodes.tolist():
            h = history[v]
            j = len(h)
            want = [sum(Fraction(h[i][t], 2 ** (j - max(i, 1))) for i in range(j)) for t in (0, 1)]
            assert [Fraction(x) for x in est[v].tolist()] == want
        prev = now
        chunk += 1
    assert chunk == (m + c_size - 1) // c_size
    assert np.all(prev[n - 3:] == -1) and np.all(st.nbr_counts()[n - 3:] == 0)
    st.close()


def test_fixed_mode_never_changes_a_label_and_keeps_first_estimates():
    rng = np.random.default_rng(3)
    n, m, c_size, P = 60, 500, 25, 33
    src = rng.integers(0, n, m).astype(np.int32)
    dst = rng.integers(0, n, m).astype(np.int32)
    seed = rng.integers(0, 2, n).astype(np.int32)
    st = oracle.EdgeStepper(src, dst, n, c_size, P, seed, oracle.EDGE_FIXED)
    prev, prev_est = st.parts(), st.nbr_counts()
    first = True
    while st.step():
        now, est = st.parts(), st.nbr_counts()
        was = prev >= 0
        assert np.array_equal(now[was], prev[was])
        if not first:
            assert np.array_equal(est[was], prev_est[was])
        nodes, fresh, prop = st.last_chunk()
        new = nodes[prev[nodes] < 0]
        assert np.array_equal(est[new], fresh[np.isin(nodes, new)].astype(np.float64))
        prev, prev_est, first = now, est, False
    st.close()


# ---------------------------------------------------------------------------------------------
# what the method is for (Sec. 4.1, 4.2): a seeded first chunk lets the stream recover a planted
# bisection, and refinement cuts fewer edges than fixed greedy decisions on small chunks
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("gseed", [0, 1])
def test_planted_bisection_refined_beats_fixed(gseed):
    g = synth.planted_partition(n=4000, blocks=2, mean_degree=12.0, seed=gseed)
    es = synth.edge_stream(g, seed=gseed + 10)
    P = oracle.capacity(g.n, 2, 1.05)
    seed = g.planted.astype(np.int32)            # only the first chunk's nodes are read
    planted_cut = oracle.edge_list_cut(es.src, es.dst, g.planted)
    cuts = {}
    for mode in (oracle.EDGE_REFINE, oracle.EDGE_FIXED):
        parts, sizes, _ = _run(es.src, es.dst, g.n, es.m // 20, P, seed, mode)
        assert sizes.max() <= P and sizes.sum() == int((parts >= 0).sum())
        cuts[mode] = oracle.edge_list_cut(es.src, es.dst, parts)
    assert cuts[oracle.EDGE_REFINE] < 0.6 * cuts[oracle.EDGE_FIXED]
    assert cuts[oracle.EDGE_REFINE] < 3.0 * planted_cut
    # one chunk holding every edge: every node is seeded, nothing else happens
    parts, sizes, est = _run(es.src, es.dst, g.n, es.m, P, seed)
    touched = np.zeros(g.n, bool)
    touched[es.src] = True
    touched[es.dst] = True
    assert np.array_equal(parts[touched], g.planted[touched]) and np.all(parts[~touched] == -1)
    deg0 = np.zeros((g.n, 2))
    np.add.at(deg0, (es.src, g.planted[es.dst]), 1)
    np.add.at(deg0, (es.dst, g.planted[es.src]), 1)
    assert np.array_equal(est, deg0)


def test_determinism_and_errors():
    rng = np.random.default_rng(9)
    n, m = 50, 200
    src = rng.integers(0, n, m).astype(np.int32)
    dst = rng.integers(0, n, m).astype(np.int32)
    seed = rng.integers(0, 2, n).astype(np.int32)
    a = _run(src, dst, n, 16, 26, seed)
    b = _run(src, dst, n, 16, 26, seed)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    with pytest.raises(oracle.OracleError) as ei:       # 2P < n
        _run(src, dst, n, 16, 24, seed)
    assert ei.value.code == oracle.ERR_ARG
    bad = seed.copy()
    bad[src[0]] = -1                                     # a first-chunk node without a seed label
    with pytest.raises(oracle.OracleError) as ei:
        _run(src, dst, n, 16, 26, bad)
    assert ei.value.code == oracle.ERR_SEED
    with pytest.raises(oracle.OracleError) as ei:       # the seed overfills a partition
        _run(src, dst, n, m, 26, np.zeros(n, np.int32))
    assert ei.value.code == oracle.ERR_SEED
    with pytest.raises(oracle.OracleError):              # endpoint out of range
        _run(np.array([0, n], np.int32), np.array([1, 2], np.int32), n, 1, 26, seed)


# ---------------------------------------------------------------------------------------------
# recursive bisection (Sec. 4.1): the driver around the two-partition procedure
# ---------------------------------------------------------------------------------------------

def _tiny_stream(rng, n, m):
    src = rng.integers(0, n, m).astype(np.int32)
    dst = rng.integers(0, n, m).astype(np.int32)
    return src, dst


def test_recursive_bisection_one_chunk_per_group_is_the_seed_bits():
    # with a single chunk every group's run consists of its seeded first chunk only: a node touched by
    # an inside edge takes its seed bit, the others alternate by size -- a closed form for the driver
    # (grouping, renumbering, inside edges, placement, 2g+b) that needs no partitioner arithmetic
    rng = np.random.default_rng(1)
    n, m, levels = 64, 90, 3
    src, dst = _tiny_stream(rng, n, m)
    # slack 2: a half may hold the whole group, so any seed bits fit
    for trial in range(5):
        bits = rng.integers(0, 2, (levels, n)).astype(np.int32)
        try:
            lab, hist = oracle.recursive_bisection(src, dst, n, levels, 1, 2.0, bits, return_levels=True)
        except oracle.OracleError:
            continue            # the random bits overfilled a half
        label = [0] * n
        for level in range(levels):
            nxt = list(label)
            for g in range(1 << level):
                mem = [v for v in range(n) if label[v] == g]
                touched = set()
                for a, b in zip(src.tolist(), dst.tolist()):
                    if label[a] == g and label[b] == g:
                        touched.add(a); touched.add(b)
                sz = [sum(1 for v in mem if v in touched and bits[level][v] == 0),
                      sum(1 for v in mem if v in touched and bits[level][v] == 1)]
                for v in mem:
                    if v in touched:
                        nxt[v] = 2 * g + int(bits[level][v])
                    else:
                        t = 1 if sz[1] < sz[0] else 0
                        sz[t] += 1
                        nxt[v] = 2 * g + t
            label = nxt
            assert hist[level].tolist() == label, (trial, level)
        return
    raise AssertionError("no trial fitted the capacity")


def test_recursive_bisection_groups_are_runs_of_the_pinned_two_partition_oracle():
    # second level rebuilt by hand from the first level's labels, with python lists, and handed to the
    # two-partition oracle that the tests above pin
    rng = np.random.default_rng(2)
    n, m, chunks, slack = 60, 400, 5, 1.2
    src, dst = _tiny_stream(rng, n, m)
    bits = np.stack([np.arange(n) % 2, (np.arange(n) // 2) % 2]).astype(np.int32)
    lab2, hist = oracle.recursive_bisection(src, dst, n, 2, chunks, slack, bits, return_levels=True)
    lab1 = oracle.recursive_bisection(src, dst, n, 1, chunks, slack, bits[:1])
    assert hist[0].tolist() == lab1.tolist()                  # deeper levels do not change earlier ones
    assert (lab2 >> 1).tolist() == lab1.tolist()
    for g in (0, 1):
        mem = [v for v in range(n) if lab1[v] == g]
        pos = {v: i for i, v in enumerate(mem)}
        sub = [(pos[a], pos[b]) for a, b in zip(src.tolist(), dst.tolist()) if a in pos and b in pos]
        s = np.array([e[0] for e in sub], np.int32)
        d = np.array([e[1] for e in sub], np.int32)
        c_size = -(-len(sub) // chunks)
        P = oracle.capacity(len(mem), 2, slack)
        parts, sizes, _ = _run(s, d, len(mem), c_size, P, bits[1][mem])
        sz = sizes.tolist()
        for i in range(len(mem)):
            if parts[i] < 0:
                t = 1 if sz[1] < sz[0] else 0
                sz[t] += 1
                parts[i] = t
        assert lab2[mem].tolist() == (2 * g + parts).tolist()
        assert max(sz) <= P and sum(sz) == len(mem)


def test_recursive_bisection_recovers_four_planted_blocks():
    g = synth.planted_partition(n=4000, blocks=4, mean_degree=14.0, seed=3)
    es = synth.edge_stream(g, seed=4)
    # seed_algo stands in as the planted block's high bit at the first level and its low bit at the second
    bits = np.stack([g.planted >> 1, g.planted & 1]).astype(np.int32)
    lab, hist = oracle.recursive_bisection(es.src, es.dst, g.n, 2, 10, 1.05, bits, return_levels=True)
    assert (hist[0] == bits[0]).mean() > 0.9
    assert (lab == g.planted).mean() > 0.8
    sizes = np.bincount(lab, minlength=4)
    assert sizes.sum() == g.n and sizes.max() <= oracle.capacity(oracle.capacity(g.n, 2, 1.05), 2, 1.05)
    assert oracle.edge_list_cut(es.src, es.dst, lab) < 2.0 * oracle.edge_list_cut(es.src, es.dst, g.planted)
    fixed = oracle.recursive_bisection(es.src, es.dst, g.n, 2, 10, 1.05, bits, oracle.EDGE_FIXED)
    assert oracle.edge_list_cut(es.src, es.dst, lab) < oracle.edge_list_cut(es.src, es.dst, fixed)


# ---------------------------------------------------------------------------------------------
# edge buckets (Sec. 3, storage layer)
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("k", [1, 2, 5])
def test_edge_buckets_against_a_bucket_by_bucket_listing(k):
    # the definition read literally: for every pair (i, j) in order, walk the stream and keep the edges
    # that go from partition i to partition j (catches a swapped pair, a transposed key, an unstable order)
    rng = np.random.default_rng(k)
    n, m = 30, 200
    src = rng.integers(0, n, m).astype(np.int32)
    dst = rng.integers(0, n, m).astype(np.int32)
    lab = rng.integers(0, k, n).astype(np.int32)
    os_, od_, off = oracle.edge_buckets(src, dst, lab, k)
    want_s, want_d, want_off = [], [], [0]
    for i in range(k):
        for j in range(k):
            for a, b in zip(src.tolist(), dst.tolist()):
                if lab[a] == i and lab[b] == j:
                    want_s.append(a); want_d.append(b)
            want_off.append(len(want_s))
    assert os_.tolist() == want_s and od_.tolist() == want_d and off.tolist() == want_off
    with pytest.raises(oracle.OracleError):
        oracle.edge_buckets(src, dst, np.full(n, k, np.int32), k)


# ---------------------------------------------------------------------------------------------
# Eq. (1): expected cuts of fixed greedy decisions from a fraction x of the edges (Sec. 4.2)
# ---------------------------------------------------------------------------------------------

def test_expected_cut_against_exact_rational_enumeration():
    # the hypergeometric tail written out with binomial coefficients in exact rationals (catches swapped
    # distribution parameters, '<=' for '<', a wrong rounding of the draws)
    from math import comb, floor
    rng = np.random.default_rng(0)
    n, m = 40, 300
    u, v = rng.integers(0, n, m), rng.integers(0, n, m)
    rowptr, colidx = synth.csr_from_pairs_np(u, v, n)
    lab = rng.integers(0, 2, n).astype(np.int32)
    for x in (0.1, 0.25, 0.5, 0.77, 1.0):
        want = Fraction(0)
        base = 0
        for i in range(n):
            nb = colidx[rowptr[i]:rowptr[i + 1]]
            c = [int((lab[nb] == 0).sum()), int((lab[nb] == 1).sum())]
            k, k0 = c[0] + c[1], max(c)
            base += k - k0
            if k == 0:
                continue
            d = min(k, floor(k * x + 0.5))
            q = Fraction(0)
            for j in range(0, d + 1):
                if 2 * j < d and j <= k0 and d - j <= k - k0:
                    q += Fraction(comb(k0, j) * comb(k - k0, d - j), comb(k, d))
            want += (k - k0) * (1 - q) + k0 * q
        got, at_one = oracle.expected_cut(rowptr, colidx, n, lab, x)
        assert at_one == base
        assert abs(got - float(want)) <= 1e-9 * max(1.0, float(want)), x
    # with every edge in hand the greedy decision is the right one: the cut seen from both ends
    got, at_one = oracle.expected_cut(rowptr, colidx, n, lab, 1.0)
    assert abs(got - at_one) < 1e-9


def test_expected_cut_falls_with_chunk_size_on_a_planted_bisection():
    g = synth.planted_partition(n=3000, blocks=2, mean_degree=16.0, seed=1)
    # from the fraction at which a typical node draws one neighbour (below it the rounded number of draws is
    # zero for most nodes and the formula counts the empty draw as a tie, i.e. as a right decision)
    vals = [oracle.expected_cut(g.rowptr, g.colidx, g.n, g.planted, x)[0] for x in (0.05, 0.1, 0.2, 0.4, 1.0)]
    assert all(a >= b - 1e-9 for a, b in zip(vals, vals[1:]))
    assert vals[0] > 1.5 * vals[-1]
    # refinement over two chunks = Eq. (1) at 2x (Sec. 4.2): fewer expected cuts than at x
    assert oracle.expected_cut(g.rowptr, g.colidx, g.n, g.planted, 0.2)[0] < vals[1]
