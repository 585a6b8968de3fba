#!/usr/bin/env python3
"""Benchmark of the GREM hot path on one MI355X.

One step = one whole `grem_partition` call (pass 0 plus the refinement passes, every chunk: row
stream, label gather, histograms, blend, arg-max, admission) on a synthetic graph that is already
resident in HBM.  Default workload: the Chung-Lu power-law graph with the vertex and edge counts of
OGBN-Papers100M (111M vertices, 1.6B directed edges, symmetrised), k=16, slack 1.05, chunk 2^20,
2 refinement passes.

Prints ONE JSON line (see the end of main).  The CPU oracle is timed beside it on a bounded sample
(`cpu_baseline`); it is a reported baseline, not the target."""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

# HBM traffic of the dominant kernels on the default workload, from two `rocprofv3 --pmc` runs
# (FETCH_SIZE, then WRITE_SIZE; KiB summed over the launches of one step, see profiles/), scaled by
# what the same counters read for a plain 2 GiB device copy (`bench.py --calibrate-copy`).  Only valid
# for the kernel sources they were taken with: `sources_sha256` is the hash of the library's sources
# at that time, and `traffic` is reported as null when the sources have changed since.
PMC = {
    "workload": "chunglu-111M",
    "sources_sha256": "d80c2ce30746ef584f9bde0885b6fb06e11bf52a7f017ac62f1b875e381130bd",
    "fetch_factor": 2.0,        # 2 GiB read  -> FETCH_SIZE 1,048,591 KiB
    "write_factor": 1.0,        # 2 GiB written -> WRITE_SIZE 2,097,152 KiB
    "fetch_kib": {"k_tp_score": 1.42675e+07, "k_tp_lookup": 1.36588e+07},
    "write_kib": {"k_tp_score": 7.32475e+06, "k_tp_lookup": 5.58938e+06},
    "launches": {"k_tp_score": 318, "k_tp_lookup": 317},
}


# The same for the edge-chunk path's dominant kernel on its 111M-node workload.
PMC_EDGE = {
    "workload": "edges-chunglu-111M-c1pct",
    "sources_sha256": "fc0898c9602363e23af93f339b153a474a59c5ea5fd2393b69a90557244403ac",
    "fetch_kib": {"k_es_count": 1.928405e+08},
    "write_kib": {"k_es_count": 9.980970e+07},
    "launches": {"k_es_count": 100},
}


def edge_sources_sha256():
    import hashlib
    with open(os.path.join(ROOT, "paper_2502_17846_amd", "csrc", "grem_edge_stream.hip"), "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()


def sources_sha256():
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2502_17846_amd", "csrc")
    # the files the two profiled kernels are compiled from
    for name in ("grem.hip", "grem_kernels.hip.h", "grem_twophase.hip.h"):
        with open(os.path.join(csrc, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic_bytes_per_chunk(workload):
    """HBM bytes one k_tp_score launch plus one k_tp_lookup launch move on average, or None."""
    if workload != PMC["workload"] or not PMC["sources_sha256"] or PMC["sources_sha256"] != sources_sha256():
        return None
    total = 0.0
    for kern in ("k_tp_score", "k_tp_lookup"):
        kib = PMC["fetch_kib"][kern] * PMC["fetch_factor"] + PMC["write_kib"][kern] * PMC["write_factor"]
        total += kib * 1024.0 / PMC["launches"][kern]
    return total

WORKLOADS = {
    # name: (generator kwargs, k, slack, chunk, refine_passes, rowptr bits)
    "chunglu-111M": dict(kind="chung_lu", n=111_000_000, m=1_600_000_000, k=16, slack=1.05,
                         chunk=1 << 20, R=2, bits=64),
    "chunglu-14M": dict(kind="chung_lu", n=13_875_000, m=200_000_000, k=16, slack=1.05,
                        chunk=1 << 17, R=2, bits=64),
    "rmat-20": dict(kind="rmat", scale=20, ef=16, k=8, slack=1.05, chunk=65_536, R=2, bits=32),
    "rmat-27": dict(kind="rmat", scale=27, ef=32, k=32, slack=1.03, chunk=1 << 22, R=1, bits=64),
    "hub-24": dict(kind="hub", scale=24, ef=16, k=256, slack=1.10, chunk=262_144, R=3, bits=32),
    "sbm-10k": dict(kind="sbm", k=4, slack=1.05, chunk=1024, R=2, bits=32),
    # Alg. 1 in the paper's own stream model (two partitions, chunks of a randomly ordered edge list);
    # c_frac is the chunk size as a fraction of the edges (Sec. 6.2 uses 1 % and 10 %)
    "edges-chunglu-111M-c1pct": dict(kind="chung_lu", n=111_000_000, m=1_600_000_000, bits=64, stream=True,
                                     c_frac=0.01, slack=1.05),
    "edges-chunglu-111M-c10pct": dict(kind="chung_lu", n=111_000_000, m=1_600_000_000, bits=64, stream=True,
                                      c_frac=0.10, slack=1.05),
    # 16 partitions by recursive bisection (Sec. 4.1, 6.2): 4 levels, every subgraph streamed in 100 chunks;
    # the per-level slack is chosen so that the compound bound equals the direct 16-way run's 1.05
    "rb-chunglu-111M-k16": dict(kind="chung_lu", n=111_000_000, m=1_600_000_000, bits=64, stream=True, levels=4,
                                chunks=100, slack=1.05 ** 0.25, direct=dict(k=16, slack=1.05, chunk=1 << 20, R=2)),
    "rb-chunglu-14M-k16": dict(kind="chung_lu", n=13_875_000, m=200_000_000, bits=64, stream=True, levels=4,
                               chunks=100, slack=1.05 ** 0.25, direct=dict(k=16, slack=1.05, chunk=1 << 17, R=2)),
    # the storage layer's edge buckets for the 16-way partition of the row-chunk path (Sec. 3)
    "buckets-chunglu-111M-k16": dict(kind="chung_lu", n=111_000_000, m=1_600_000_000, bits=64, stream=True, buckets=True,
                                     direct=dict(k=16, slack=1.05, chunk=1 << 20, R=2)),
    "buckets-chunglu-14M-k16": dict(kind="chung_lu", n=13_875_000, m=200_000_000, bits=64, stream=True, buckets=True,
                                    direct=dict(k=16, slack=1.05, chunk=1 << 17, R=2)),
    # Eq. (1) of Sec. 4.2 evaluated for a two-way labelling of the bench graph at x = 1 %
    "eq1-chunglu-111M": dict(kind="chung_lu", n=111_000_000, m=1_600_000_000, bits=64, eq1=True, x=0.01),
    "eq1-chunglu-14M": dict(kind="chung_lu", n=13_875_000, m=200_000_000, bits=64, eq1=True, x=0.01),
    "edges-chunglu-14M-c1pct": dict(kind="chung_lu", n=13_875_000, m=200_000_000, bits=64, stream=True,
                                    c_frac=0.01, slack=1.05),
}


def make_graph(w, device):
    import torch
    from paper_2502_17846_amd import synth
    rdt = torch.int64 if w["bits"] == 64 else torch.int32
    if w["kind"] == "chung_lu":
        return synth.chung_lu(w["n"], w["m"], gamma=2.1, cap=50_000.0, seed=0, device=device,
                              rowptr_dtype=rdt)
    if w["kind"] == "rmat":
        return synth.rmat(w["scale"], w["ef"], seed=0, device=device, rowptr_dtype=rdt)
    if w["kind"] == "hub":
        return synth.hub_stress(w["scale"], w["ef"], hubs=64, hub_degree=2_000_000, seed=0,
                                device=device, rowptr_dtype=rdt)
    if w["kind"] == "sbm":
        g = synth.planted_partition(seed=0)
        g.rowptr = torch.as_tensor(g.rowptr).to(device)
        g.colidx = torch.as_tensor(g.colidx).to(device)
        return g
    raise ValueError(w["kind"])


def algorithmic_bytes(n, nnz, k, R, rowptr_bytes, label_bytes):
    """Bytes GREM itself must move per run: per pass the row offsets and column ids once, E written
    (pass 0) or read and written (later passes), compact labels read and written once.  The label
    gathers are served from cache and are not counted."""
    common = rowptr_bytes * (n + 1) + 4 * nnz + 2 * label_bytes * n
    first = common + 4 * n * k
    later = common + 8 * n * k
    return first, later, first + R * later


def emit(out):
    """Prints the one JSON line; the host the oracle ran on goes beside its rate."""
    if isinstance(out.get("cpu_baseline"), dict) and "cpu_model" not in out["cpu_baseline"]:
        out["cpu_baseline"].update(host_info())
    print(json.dumps(out))


def host_info():
    """CPU model and core count of the host the oracle is timed on."""
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return {"cpu_model": model, "nproc": os.cpu_count()}


def cpu_baseline(g, w, budget_s=9.0, max_chunks=24):
    """The oracle, single thread, on the first chunks of the same graph: a sample of pass 0, and a sample of
    a refinement pass.  The rows after the sample are left empty, so that the oracle gets through the rest of
    pass 0 quickly (untimed) and the sample's rows can be refined with every vertex labelled."""
    import numpy as np
    import torch
    import oracle
    n, chunk, R = g.n, w["chunk"], w["R"]
    nchunks = (n + chunk - 1) // chunk
    m = min(max_chunks, nchunks)
    rows = min(n, m * chunk)
    rp_full = g.rowptr.to(torch.int64)
    end = int(rp_full[rows].item())
    rp_host = rp_full.cpu().numpy().copy()
    rp_host[rows:] = end                        # rows after the sample are left empty
    ci_host = g.colidx[:end].cpu().numpy()
    st = oracle.Stepper(rp_host, ci_host, n, w["k"], w["slack"], chunk, min(R, 1))
    done0, t0 = 0, time.perf_counter()
    while done0 < m:
        st.step()
        done0 += 1
        if time.perf_counter() - t0 > budget_s:
            break
    dt0 = time.perf_counter() - t0
    entries0 = int(rp_host[min(n, done0 * chunk)])
    rate0 = entries0 / dt0
    rate1, done1, dt1, entries1 = None, 0, 0.0, 0
    if R >= 1:
        while st.position[0] == 0:              # the rest of pass 0: rows without entries (untimed)
            st.step()
        t1 = time.perf_counter()
        while done1 < done0:
            st.step()
            done1 += 1
            if time.perf_counter() - t1 > budget_s:
                break
        dt1 = time.perf_counter() - t1
        entries1 = int(rp_host[min(n, done1 * chunk)])
        rate1 = entries1 / dt1
    st.close()
    # CSR entries per second averaged over the passes of one step (pass 0 once, a refinement pass R times)
    per_entry = (1.0 / rate0 + (R / rate1 if rate1 else 0.0)) / (R + 1 if rate1 else 1)
    entries_per_s = 1.0 / per_entry
    out = {
        "value": entries_per_s * (g.directed_edges / g.nnz), "unit": "edges/s per pass", "cores": 1, "kind": "oracle",
        "sample": f"the first {done0} of {nchunks} chunks ({entries0} CSR entries) of the same graph in pass 0, "
                  f"{dt0:.1f} s" + (f"; the first {done1} chunks ({entries1} entries) in a refinement pass, {dt1:.1f} s "
                                    f"(rows after the sample left empty, every vertex labelled)" if rate1 else "")
                  + f"; label table and estimates of all {n} vertices; averaged over 1 + {R} passes",
        "csr_entries_per_s": entries_per_s,
        "pass0_csr_entries_per_s": rate0,
        "refine_pass_csr_entries_per_s": rate1,
    }
    out.update(host_info())
    return out


def copy_bandwidth_gbps(dev, nbytes=4 << 30, reps=5):
    """Measured rate of a plain device-to-device copy (bytes read plus bytes written per second)."""
    import torch
    a = torch.empty(nbytes // 4, dtype=torch.int32, device=dev).fill_(1)
    b = torch.empty_like(a)
    b.copy_(a)
    torch.cuda.synchronize()
    best = None
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        b.copy_(a)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        best = ms if best is None or ms < best else best
    del a, b
    torch.cuda.empty_cache()
    return 2.0 * nbytes / (best * 1e-3) / 1e9


def bench_edge_stream(args, w, dev):
    """The edge-chunk path: a step is one whole run of Alg. 1 over the stream (every chunk once)."""
    import numpy as np
    import torch
    from paper_2502_17846_amd import binding as B
    from paper_2502_17846_amd import synth
    t_gen = time.perf_counter()
    g = make_graph(w, dev)
    es = synth.edge_stream(g, seed=1)
    n, m = es.n, es.m
    gname = g.name
    del g
    torch.cuda.empty_cache()
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen
    c_size = max(1, int(round(m * w["c_frac"])))
    nchunks = (m + c_size - 1) // c_size
    P = B.grem_capacity(n, 2, w["slack"])
    # stands for seed_algo's output on the first chunk: id parity, balanced by construction
    seed = (torch.arange(n, device=dev, dtype=torch.int32) & 1)
    print(f"[bench] {es.name}: n={n} edges={m} c_size={c_size} ({nchunks} chunks) generated in {t_gen:.1f}s",
          file=sys.stderr, flush=True)
    est = torch.empty((n, 2), dtype=torch.float64, device=dev)
    out_parts = [None]

    def step():
        lib = B.load()
        parts = torch.empty(n, dtype=torch.int32, device=dev)
        rc = lib.grem_edge_stream_bipartition(es.src.data_ptr(), es.dst.data_ptr(), m, n, c_size, P,
                                              seed.data_ptr(), B.EDGE_REFINE, parts.data_ptr(), None,
                                              est.data_ptr(), torch.cuda.current_stream().cuda_stream)
        if rc != 0:
            raise RuntimeError(f"grem_edge_stream_bipartition returned {rc}")
        out_parts[0] = parts

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    parts = out_parts[0]
    cut = int(B.grem_edge_list_cut(es.src, es.dst, parts).item())
    assigned = parts >= 0
    sizes = torch.bincount(parts[assigned], minlength=2)
    assert int(sizes.max()) <= P

    # dominant kernel: k_es_count reads each edge's two ids once (8 bytes); its label look-ups and count
    # atomics are random accesses whose useful bytes are 2 and 16 per edge
    roofline = {"bound": "hbm", "achieved": None, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": None,
                "traffic": None, "kernel": "k_es_count"}
    if not args.no_kernel_timing:
        B.grem_edge_stream_profile_enable(True)
        step()
        torch.cuda.synchronize()
        count_ms, launches, _ = B.grem_edge_stream_profile_read()
        B.grem_edge_stream_profile_enable(False)
        bytes_per_launch = 8.0 * m / launches
        avg_s = 1e-3 * count_ms / launches
        achieved = bytes_per_launch / avg_s / 1e9
        roofline.update(achieved=achieved, frac=achieved / HBM_PEAK_GBPS, avg_launch_us=1e6 * avg_s,
                        launches_per_step=launches, bytes_per_launch=bytes_per_launch,
                        count_ms_per_step=round(count_ms, 3))
        if args.workload == PMC_EDGE["workload"] and PMC_EDGE["sources_sha256"] == edge_sources_sha256():
            kib = (PMC_EDGE["fetch_kib"]["k_es_count"] * PMC["fetch_factor"]
                   + PMC_EDGE["write_kib"]["k_es_count"] * PMC["write_factor"])
            roofline["traffic"] = kib * 1024.0 / PMC_EDGE["launches"]["k_es_count"]
    out = {
        "metric": "edges/sec per GREM pass", "value": m / (elapsed / args.steps), "unit": "edges/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {es.name} of {gname}; two partitions, c_size={c_size} "
                               f"({100 * w['c_frac']:g} % of the edges), P={P}, first chunk seeded by id parity",
                   "n": n, "edges": m, "chunks_per_step": nchunks},
        "cut_fraction": cut / m, "sizes": sizes.tolist(), "capacity": P,
        "unassigned_nodes": int((~assigned).sum()),
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        import oracle
        print("[bench] timing the CPU oracle on a sample ...", file=sys.stderr, flush=True)
        take = min(nchunks, 12)
        ms_ = min(m, take * c_size)
        hs, hd = es.src[:ms_].cpu().numpy(), es.dst[:ms_].cpu().numpy()
        st = oracle.EdgeStepper(hs, hd, n, c_size, P, seed.cpu().numpy())
        done, t0 = 0, time.perf_counter()
        while done < take and st.step():
            done += 1
            if time.perf_counter() - t0 > 15.0:
                break
        dt = time.perf_counter() - t0
        st.close()
        out["cpu_baseline"] = {"value": min(ms_, done * c_size) / dt, "unit": "edges/s", "cores": 1, "kind": "oracle",
                               "sample": f"first {done} of {nchunks} chunks ({min(ms_, done * c_size)} edges) of the "
                                         f"same stream, {dt:.1f} s, state for all {n} nodes"}
    emit(out)


def bench_eq1(args, w, dev):
    """Eq. (1): a step is one evaluation of E[C](x) over the whole graph."""
    import numpy as np
    import torch
    from paper_2502_17846_amd import binding as B
    g = make_graph(w, dev)
    n, nnz, x = g.n, g.nnz, w["x"]
    labels = (torch.arange(n, device=dev, dtype=torch.int32) & 1)     # any two-way labelling is a valid input
    res = [None]

    def step():
        res[0] = B.grem_expected_cut(g.rowptr, g.colidx, n, labels, x)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / args.steps
    ec, base = res[0].cpu().numpy().tolist()
    # algorithmic bytes: row offsets, column ids and labels once (the label look-ups would be cache traffic)
    nbytes = (w["bits"] // 8) * (n + 1) + 4 * nnz + 4 * n
    out = {
        "metric": "edges/sec per GREM pass", "value": g.directed_edges / sec, "unit": "edges/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": 1e3 * sec, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {g.name}; Eq. (1) at x={x} for the id-parity labelling", "n": n,
                   "csr_entries": nnz},
        "expected_cut_fraction": ec / nnz, "cut_fraction_at_x_1": base / nnz,
        "roofline": {"bound": "hbm", "achieved": nbytes / sec / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": nbytes / sec / 1e9 / HBM_PEAK_GBPS, "traffic": None, "kernel": "k_xc_terms"},
    }
    if not args.no_kernel_timing:
        # the same evaluation, and the cut, on a plan of the graph (label look-ups served from LDS)
        def timed(f, reps=5):
            f()
            torch.cuda.synchronize()
            ts = []
            for _ in range(reps):
                t0 = time.perf_counter()
                r = f()
                torch.cuda.synchronize()
                ts.append(1e3 * (time.perf_counter() - t0))
            return r, sorted(ts)[len(ts) // 2]
        t0 = time.perf_counter()
        plan = B.Plan(g.rowptr, g.colidx, n, 1 << 20)
        torch.cuda.synchronize()
        plan_ms = 1e3 * (time.perf_counter() - t0)
        with plan:
            # the calls' state from a workspace, as in the partition bench (stream-ordered allocations of
            # several GB per call would be most of the time)
            ws = torch.empty(plan.call_bytes(2, 0, seeded=True, with_estimates_out=True) + 8 * n + 4096,
                             dtype=torch.uint8, device=dev)
            B.grem_set_workspace(ws)
            try:
                pe, pe_ms = timed(lambda: B.grem_plan_expected_cut(plan, labels, x))
                pc, pc_ms = timed(lambda: B.grem_plan_edge_cut(plan, 2, labels))
            finally:
                B.grem_set_workspace(None)
            cc, cc_ms = timed(lambda: B.grem_edge_cut(g.rowptr, g.colidx, n, labels))
        pec, pbase = pe.cpu().numpy().tolist()
        assert pbase == base and abs(pec - ec) <= 1e-9 * ec and int(pc.item()) == int(cc.item())
        out["on_a_plan"] = {"plan_create_ms": round(plan_ms, 3), "expected_cut_ms": round(pe_ms, 3),
                            "edge_cut_ms": round(pc_ms, 3), "edge_cut_csr_walk_ms": round(cc_ms, 3),
                            "is": "grem_plan_expected_cut / grem_plan_edge_cut on a grem_plan of the same graph "
                                  "(median of 5), equal to the CSR routines' results"}
    if not args.no_cpu_baseline:
        import oracle
        rows = min(n, 2_000_000)
        rp = g.rowptr[:rows + 1].cpu().numpy()
        end = int(rp[-1])
        rp_full = np.concatenate([rp, np.full(n - rows, end, dtype=rp.dtype)])
        ci = g.colidx[:end].cpu().numpy()
        t0 = time.perf_counter()
        oracle.expected_cut(rp_full, ci, n, labels.cpu().numpy(), x)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": end * (g.directed_edges / nnz) / dt, "unit": "edges/s", "cores": 1,
                               "kind": "oracle", "sample": f"the first {rows} rows ({end} CSR entries) of the same graph, "
                                                           f"labels of all {n} nodes, {dt:.1f} s"}
    emit(out)


def bench_buckets(args, w, dev):
    """Edge buckets of a partitioned graph: a step is one grouping of the whole edge list."""
    import torch
    from paper_2502_17846_amd import binding as B
    from paper_2502_17846_amd import synth
    g = make_graph(w, dev)
    es = synth.edge_stream(g, seed=1)
    d = w["direct"]
    n, m, k = es.n, es.m, d["k"]
    lab = B.grem_partition(g.rowptr, g.colidx, n, k, d["slack"], d["chunk"], d["R"])
    del g
    torch.cuda.empty_cache()
    torch.cuda.synchronize()
    print(f"[bench] {es.name}: n={n} edges={m} k={k}", file=sys.stderr, flush=True)
    res = [None]

    def step():
        res[0] = B.grem_edge_buckets(es.src, es.dst, n, lab, k)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    out_s, out_d, off = res[0]
    sizes = (off[1:] - off[:-1]).reshape(k, k)
    assert int(off[-1]) == m
    # algorithmic bytes of the whole grouping: every edge read once and written once (8 + 8 bytes)
    sec = elapsed / args.steps
    out = {
        "metric": "edges/sec per GREM pass", "value": m / sec, "unit": "edges/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": 1e3 * sec, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {es.name}; edge buckets for the {k}-way partition of the row-chunk "
                               f"path ({d})", "n": n, "edges": m, "buckets": k * k},
        "uncut_fraction": float(sizes.diag().sum()) / m,
        "largest_bucket": int(sizes.max()), "smallest_bucket": int(sizes.min()),
        "roofline": {"bound": "hbm", "achieved": 16.0 * m / sec / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": 16.0 * m / sec / 1e9 / HBM_PEAK_GBPS, "traffic": None,
                     "kernel": "whole call (k_eb_hist + k_eb_scatter and the scans, timed together)"},
    }
    if not args.no_cpu_baseline:
        import oracle
        take = min(m, 30_000_000)
        hs, hd, hl = es.src[:take].cpu().numpy(), es.dst[:take].cpu().numpy(), lab.cpu().numpy()
        t0 = time.perf_counter()
        oracle.edge_buckets(hs, hd, hl, k)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": take / dt, "unit": "edges/s", "cores": 1, "kind": "oracle",
                               "sample": f"the first {take} edges of the same stream with the same labels, {dt:.1f} s"}
    emit(out)


def bench_recursive(args, w, dev):
    """2^levels partitions by recursive bisection: a step is the whole recursion."""
    import torch
    from paper_2502_17846_amd import binding as B
    from paper_2502_17846_amd import synth
    t_gen = time.perf_counter()
    g = make_graph(w, dev)
    es = synth.edge_stream(g, seed=1)
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen
    n, m, levels, chunks = es.n, es.m, w["levels"], w["chunks"]
    ids = torch.arange(n, device=dev, dtype=torch.int32)
    seed_bits = torch.stack([(ids >> l) & 1 for l in range(levels)]).contiguous()   # stands for seed_algo
    print(f"[bench] {es.name}: n={n} edges={m} levels={levels} chunks={chunks} generated in {t_gen:.1f}s",
          file=sys.stderr, flush=True)
    out_lab = [None]

    def step():
        out_lab[0] = B.grem_recursive_bisection(es.src, es.dst, n, levels, chunks, w["slack"], seed_bits.reshape(-1))

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    lab = out_lab[0]
    k = 1 << levels
    sizes = torch.bincount(lab, minlength=k)
    cut = int(B.grem_edge_list_cut(es.src, es.dst, lab).item())
    roofline = {"bound": "hbm", "achieved": None, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": None,
                "traffic": None, "kernel": "k_es_count"}
    if not args.no_kernel_timing:
        B.grem_edge_stream_profile_enable(True)
        step()
        torch.cuda.synchronize()
        count_ms, launches, streamed = B.grem_edge_stream_profile_read()
        B.grem_edge_stream_profile_enable(False)
        # algorithmic bytes of k_es_count: the two ids of every edge it is handed
        bytes_per_launch = 8.0 * streamed / launches
        avg_s = 1e-3 * count_ms / launches
        achieved = bytes_per_launch / avg_s / 1e9
        roofline.update(achieved=achieved, frac=achieved / HBM_PEAK_GBPS, avg_launch_us=1e6 * avg_s,
                        launches_per_step=launches, bytes_per_launch=bytes_per_launch,
                        count_ms_per_step=round(count_ms, 3), edges_streamed_per_step=streamed)
    # the direct k-way run of the row-chunk path on the same graph, for the cut comparison
    d = w["direct"]
    dlab = B.grem_partition(g.rowptr, g.colidx, n, d["k"], d["slack"], d["chunk"], d["R"])
    dcut = int(B.grem_edge_list_cut(es.src, es.dst, dlab).item())
    torch.cuda.synchronize()
    out = {
        "metric": "edges/sec per GREM pass",
        "value": (roofline.get("edges_streamed_per_step") or m * levels) / (elapsed / args.steps), "unit": "edges/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": 1e3 * elapsed / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {es.name}; {k} partitions by {levels} levels of bisection, "
                               f"{chunks} chunks per subgraph, slack {w['slack']:.5f} per level, seeds = id bits",
                   "n": n, "edges": m, "levels": levels},
        "note": "value counts the edges actually streamed over all levels (edges cut at a level leave the stream)",
        "cut_fraction": cut / m, "max_partition_size": int(sizes.max()), "min_partition_size": int(sizes.min()),
        "direct_kway": {"cut_fraction": dcut / m, "config": d,
                        "max_partition_size": int(torch.bincount(dlab, minlength=k).max())},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        import oracle
        c_size = (m + chunks - 1) // chunks
        take = min(chunks, 12)
        ms_ = min(m, take * c_size)
        st = oracle.EdgeStepper(es.src[:ms_].cpu().numpy(), es.dst[:ms_].cpu().numpy(), n, c_size,
                                B.grem_capacity(n, 2, w["slack"]), seed_bits[0].cpu().numpy())
        done, t0 = 0, time.perf_counter()
        while done < take and st.step():
            done += 1
            if time.perf_counter() - t0 > 15.0:
                break
        dt = time.perf_counter() - t0
        st.close()
        out["cpu_baseline"] = {"value": min(ms_, done * c_size) / dt, "unit": "edges/s", "cores": 1, "kind": "oracle",
                               "sample": f"first level only: first {done} of {chunks} chunks ({min(ms_, done * c_size)} edges) of "
                                         f"the same stream, {dt:.1f} s (the recursion's oracle runs the same stepper per group)"}
    emit(out)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="chunglu-111M", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true",
                    help="skip the extra instrumented steps (per-pass and per-kernel times, the planned call)")
    ap.add_argument("--no-copy-bandwidth", action="store_true", help="skip the device-copy rate measurement")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a plain device copy of 2 GiB (8 launches): under rocprofv3 --pmc its "
                         "FETCH_SIZE / WRITE_SIZE give the factor that scales those counters to bytes")
    ap.add_argument("--col-bits", type=int, default=0,
                    help="log2 of the vertices per column block of the two-phase path (0 = library default)")
    ap.add_argument("--hub-degree", type=int, default=0,
                    help="degree from which a row is spread over the chunk's workgroups (0 = library default)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU; run with --gpus 1 "
              "(the partitioner has no multi-GPU path)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2502_17846_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    if args.calibrate_copy:
        nbytes = 2 << 30
        a = torch.ones(nbytes // 4, dtype=torch.int32, device=dev)
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        for _ in range(8):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "device copy", "bytes_read_per_launch": nbytes,
                          "bytes_written_per_launch": nbytes, "launches": 8}))
        return
    w = WORKLOADS[args.workload]
    if w.get("eq1"):
        bench_eq1(args, w, dev)
        return
    if w.get("buckets"):
        bench_buckets(args, w, dev)
        return
    if w.get("levels"):
        bench_recursive(args, w, dev)
        return
    if w.get("stream"):
        bench_edge_stream(args, w, dev)
        return
    t_gen = time.perf_counter()
    g = make_graph(w, dev)
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen
    n, nnz, k, R, chunk = g.n, g.nnz, w["k"], w["R"], w["chunk"]
    print(f"[bench] {g.name}: n={n} nnz={nnz} directed={g.directed_edges} generated in {t_gen:.1f}s",
          file=sys.stderr, flush=True)

    opts = B.options(col_bits=args.col_bits, hub_degree=args.hub_degree) if (args.col_bits or args.hub_degree) else None
    plan_opts = B.options(col_bits=args.col_bits, hub_degree=args.hub_degree, plan_max_k=k if k > 16 else 0)
    ws_bytes = B.grem_workspace_bytes_two_phase(n, nnz, k, chunk, opts)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    B.grem_set_workspace(ws)
    labels = torch.empty(n, dtype=torch.int32, device=dev)

    def step():
        B.grem_partition(g.rowptr, g.colidx, n, k, w["slack"], chunk, R, labels_out=labels, options=opts)

    def timed(fn, reps):
        """Each repetition bracketed by a device synchronisation; milliseconds per repetition."""
        out = []
        for _ in range(reps):
            torch.cuda.synchronize()
            t = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            out.append(1e3 * (time.perf_counter() - t))
        return out

    def stats(ms):
        srt = sorted(ms)
        return {"median_ms": srt[len(srt) // 2] if len(srt) % 2 else 0.5 * (srt[len(srt) // 2 - 1] + srt[len(srt) // 2]),
                "min_ms": srt[0], "mean_ms": sum(srt) / len(srt), "repetitions": len(srt)}

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    per_step = timed(step, args.steps)
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    passes = R + 1
    sec_per_pass = elapsed / (args.steps * passes)
    edges_per_s = g.directed_edges / sec_per_pass

    # result summary (also a cheap sanity check of the run that was timed)
    cut = int(B.grem_edge_cut(g.rowptr, g.colidx, n, labels).item())
    sizes = torch.bincount(labels, minlength=k)
    P = B.grem_capacity(n, k, w["slack"])
    assert int(sizes.max()) <= P and int(sizes.sum()) == n and int(labels.min()) >= 0

    label_bytes = 1 if k <= 255 else 2
    b_first, b_later, b_total = algorithmic_bytes(n, nnz, k, R, w["bits"] // 8, label_bytes)
    nchunks = (n + chunk - 1) // chunk
    frac_of_peak = lambda nbytes, ms: nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS
    roofline = {"bound": "hbm", "achieved": None, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": None,
                "traffic": None, "kernel": "k_score_lds" if k <= 128 else "k_score_global",
                "frac_is": "the dominant kernel's: algorithmic bytes of one chunk / its average launch time",
                "whole_call_frac": frac_of_peak(b_total, ms_per_step),
                "whole_call_frac_is": "algorithmic bytes of all passes / ms_per_step (validation, re-layout and "
                                      "every kernel of every chunk included)"}

    def per_pass_marks(fn):
        """[ms before the first pass, pass 0, ..., pass R, output expansion] of one call, from events at the passes'
        boundaries on the caller's stream."""
        B.grem_profile_enable(1)
        B.grem_profile_reset()
        fn()
        torch.cuda.synchronize()
        marks = B.grem_profile_read_marks()
        B.grem_profile_enable(0)
        B.grem_profile_reset()
        return marks

    def pass_report(marks):
        # marks: call start .. (plan) .. first pass | passes | outputs; the passes are the R + 1 before the last
        p = marks[-(passes + 1):-1]
        rep = {"before_first_pass_ms": round(sum(marks[:-(passes + 1)]), 4), "pass_ms": [round(x, 4) for x in p],
               "after_last_pass_ms": round(marks[-1], 4),
               "pass0_frac": frac_of_peak(b_first, p[0]),
               "pass0_csr_entries_per_s": nnz / (p[0] * 1e-3)}
        if R >= 1:
            later = sorted(p[1:])
            med = later[len(later) // 2]
            rep.update(refine_pass_median_ms=round(med, 4), refine_pass_frac=frac_of_peak(b_later, med),
                       refine_pass_csr_entries_per_s=nnz / (med * 1e-3))
        return rep

    planned = None
    if not args.no_kernel_timing:
        roofline["cold_call"] = pass_report(per_pass_marks(step))
        B.grem_profile_enable(2)
        B.grem_profile_reset()
        step()
        torch.cuda.synchronize()
        score_ms, score_launches = B.grem_profile_read(B.KERNEL_SCORE)
        per_class = {}
        for c in range(B.KERNEL_CLASSES):
            ms, cnt = B.grem_profile_read(c)
            per_class[B.kernel_name(c)] = {"ms": round(ms, 4), "launches": cnt}
        B.grem_profile_enable(0)
        B.grem_profile_reset()
        # On the two-phase path the score of a chunk is two launches: the histogram/blend/arg-max
        # kernel and the look-up kernel that prepares the next chunks' input; they are timed as one.
        lookup_ms = per_class.get("lookup", {}).get("ms", 0.0)
        two_phase = per_class.get("lookup", {}).get("launches", 0) > 0
        if two_phase:
            roofline["kernel"] = "k_tp_score+k_tp_lookup"
            roofline["score_ms"], roofline["lookup_ms"] = round(score_ms, 4), round(lookup_ms, 4)
            roofline["traffic"] = measured_traffic_bytes_per_chunk(args.workload)
            roofline["relayout_ms"] = round(per_class.get("relayout", {}).get("ms", 0.0), 4)
        bytes_per_launch = b_total / (passes * nchunks)
        avg_launch_s = 1e-3 * (score_ms + lookup_ms) / max(score_launches, 1)
        achieved = bytes_per_launch / avg_launch_s / 1e9
        roofline.update(achieved=achieved, frac=achieved / HBM_PEAK_GBPS,
                        avg_launch_us=1e6 * avg_launch_s, launches_per_step=score_launches,
                        bytes_per_launch=bytes_per_launch, per_kernel_class_ms=per_class)
        if two_phase:
            # the same run on a plan: the re-laid-out copy is built once per graph and kept
            B.grem_set_workspace(None)
            del ws
            torch.cuda.empty_cache()
            t_plan = time.perf_counter()
            plan = B.Plan(g.rowptr, g.colidx, n, chunk, plan_opts)
            torch.cuda.synchronize()
            t_plan = 1e3 * (time.perf_counter() - t_plan)
            plabels = torch.empty(n, dtype=torch.int32, device=dev)
            pws = torch.empty(plan.call_bytes(k, R), dtype=torch.uint8, device=dev)
            B.grem_set_workspace(pws)

            def pstep():
                B.grem_partition_planned(plan, k, w["slack"], R, labels_out=plabels)

            for _ in range(max(1, args.warmup)):
                pstep()
            pms = timed(pstep, args.steps)
            assert torch.equal(plabels, labels)
            planned = stats(pms)
            planned.update(plan_create_ms=round(t_plan, 3), plan_device_bytes=plan.device_bytes,
                           call_workspace_bytes=pws.numel(),
                           value=g.directed_edges / (planned["mean_ms"] * 1e-3 / passes), unit="edges/s",
                           whole_call_frac=frac_of_peak(b_total, planned["mean_ms"]))
            planned.update(pass_report(per_pass_marks(pstep)))
            roofline["planned_call_frac"] = planned["whole_call_frac"]
            B.grem_set_workspace(None)
            plan.close()

    out = {
        "metric": "edges/sec per GREM pass",
        "value": edges_per_s,
        "unit": "edges/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: {g.name}, k={k}, slack={w['slack']}, chunk={chunk}, "
                               f"refine_passes={R}", "n": n, "csr_entries": nnz,
                   "directed_edges": g.directed_edges, "passes_per_step": passes,
                   "chunks_per_pass": nchunks},
        "step_is": "one whole grem_partition call on a graph it has not seen: validation, re-layout of the entries, "
                   "pass 0 and the refinement passes",
        "step_ms": stats(per_step),
        "csr_entries_per_s": nnz / sec_per_pass,
        "ms_per_pass": 1e3 * sec_per_pass,
        "algorithmic_GB_per_step": b_total / 1e9,
        "algorithmic_GB_pass0": b_first / 1e9,
        "algorithmic_GB_refine_pass": b_later / 1e9,
        "whole_step_algorithmic_GBps": b_total / (elapsed / args.steps) / 1e9,
        "workspace_bytes": ws_bytes,
        "cut_fraction": cut / max(nnz, 1),
        "max_partition_size": int(sizes.max()),
        "capacity": P,
        "roofline": roofline,
    }
    if planned is not None:
        out["planned_call"] = planned
        out["planned_call_is"] = ("grem_partition_planned on a grem_plan of the same graph (the re-laid-out copy built "
                                  "once by grem_plan_create, plan_create_ms, and kept): the passes alone")
    B.grem_set_workspace(None)
    if not args.no_copy_bandwidth:
        bw = copy_bandwidth_gbps(dev)
        out["device_copy_GBps"] = bw
        roofline["whole_call_frac_of_copy_rate"] = b_total / (ms_per_step * 1e-3) / 1e9 / bw
    if not args.no_cpu_baseline:
        print("[bench] timing the CPU oracle on a sample ...", file=sys.stderr, flush=True)
        out["cpu_baseline"] = cpu_baseline(g, w)
    emit(out)


if __name__ == "__main__":
    main()
