"""The C-ABI library loads and exports every symbol that include/grem.h declares (no compute
calls: this runs without a GPU), and the host-only helpers agree with the paper's definitions."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "grem.h")
LIB = os.path.join(ROOT, "paper_2502_17846_amd", "libgrem.so")


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(grem_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2502_17846_amd import build
        build.build_library()
    return ctypes.CDLL(LIB)


def test_header_declares_the_boundary():
    names = _declared()
    for must in ("grem_partition", "grem_partition_seeded", "grem_edge_cut", "grem_capacity",
                 "grem_workspace_bytes", "grem_set_workspace", "grem_status_string"):
        assert must in names


def test_library_exports_every_declared_symbol(lib):
    for name in _declared():
        assert hasattr(lib, name), name


def test_binding_lists_the_same_names():
    from paper_2502_17846_amd import binding
    assert sorted(binding.EXPORTS) == _declared()


def test_host_helpers(lib):
    lib.grem_capacity.restype = ctypes.c_int64
    lib.grem_capacity.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_double]
    # balanced objective ceil(V/p) of Sec. 4.1, widened by the slack
    assert lib.grem_capacity(10, 3, 1.0) == 4
    assert lib.grem_capacity(10_000, 4, 1.05) == 2625
    assert lib.grem_capacity(111_000_000, 16, 1.05) == 7_284_375
    assert lib.grem_capacity(1 << 24, 256, 1.10) == 72_090
    assert lib.grem_capacity(0, 4, 1.05) == -1
    assert lib.grem_capacity(10, 4, 0.5) == -1
    lib.grem_workspace_bytes.restype = ctypes.c_size_t
    lib.grem_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int64]
    lib.grem_workspace_bytes_two_phase.restype = ctypes.c_size_t
    lib.grem_workspace_bytes_two_phase.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int32, ctypes.c_int64,
                                                   ctypes.c_void_p]
    n, nnz, k, chunk = 1 << 20, 30_000_000, 8, 1 << 16
    # plain route: E, compact labels, the chunk's proposals and small tables
    w = lib.grem_workspace_bytes(n, k, chunk)
    assert n * k * 4 + n <= w < n * k * 4 + 2 * n + (1 << 20)
    w64 = lib.grem_workspace_bytes(n, 64, chunk)
    assert n * 64 * 4 + n <= w64 < n * 64 * 4 + 2 * n + (1 << 20)
    # two-phase route: the re-laid-out entries (3 + 2 bytes each) and, taking turns in one region, the 4-byte
    # intermediate copy and the per-call state; offset tables on top
    w2 = lib.grem_workspace_bytes_two_phase(n, nnz, k, chunk, None)
    assert w2 >= n + 9 * nnz and w2 < 20 * n + 9 * nnz + (96 << 20)
    assert lib.grem_workspace_bytes_two_phase(n, nnz, 64, chunk, None) == w64      # no entry copy above k = 16
    assert lib.grem_workspace_bytes(0, k, chunk) == 0
    assert lib.grem_workspace_bytes_two_phase(0, nnz, k, chunk, None) == 0
    # the bench workload: less than three times the 13.7 GB of its CSR
    assert lib.grem_workspace_bytes_two_phase(111_000_000, 3_193_913_564, 16, 1 << 20, None) < 40e9
    lib.grem_status_string.restype = ctypes.c_char_p
    assert lib.grem_status_string(0) == b"ok"
    assert b"seed" in lib.grem_status_string(-5)


def test_capacity_matches_oracle_on_a_grid(lib):
    import oracle
    lib.grem_capacity.restype = ctypes.c_int64
    lib.grem_capacity.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_double]
    for n in (1, 7, 1000, 10_000, 999_983, 1 << 20, 111_000_000, (1 << 31) - 1):
        for k in (1, 2, 3, 16, 100, 256, 4096):
            for slack in (1.0, 1.01, 1.03, 1.05, 1.1, 1.5, 2.0):
                assert lib.grem_capacity(n, k, slack) == oracle.capacity(n, k, slack)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""
