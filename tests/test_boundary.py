"""CPU-side checks of the boundary: the C-ABI library builds for gfx950, loads
without a GPU and exports every entry point that include/dct.h declares; the
Python binding marshals the same names.  No kernel is launched here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_entry_points():
    text = open(os.path.join(ROOT, "include", "dct.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dct_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_four_calls():
    names = declared_entry_points()
    for want in ("dct_select_threshold", "dct_threshold_compact", "dct_rowtopk_fwd", "dct_rowtopk_bwd"):
        assert want in names


def test_library_exports_every_declared_symbol():
    import paper_2010_08899_amd as m
    from paper_2010_08899_amd import binding, build
    handle = m.lib()
    assert os.path.exists(build.LIB)
    raw = ctypes.CDLL(build.LIB)
    for name in declared_entry_points():
        assert hasattr(raw, name), name
        assert name in binding._EXPORTS, name
        assert hasattr(m, name), name
    assert handle.dct_status_string(0) == b"DCT_OK"
    # the benchmark's streaming probes are not part of the product library or its header
    assert not hasattr(raw, "dct_probe_read") and not hasattr(raw, "dct_bench_probe_read")
    bench = ctypes.CDLL(build.BENCH_LIB)
    assert all(hasattr(bench, f"dct_bench_probe_{p}") for p in ("read", "copy", "rows"))


def test_host_side_argument_checks_need_no_gpu():
    import paper_2010_08899_amd as m
    lib = m.lib()
    assert m.dct_select_threshold_workspace_bytes(m.DCT_F32, 0) == 0
    assert m.dct_select_threshold_workspace_bytes(m.DCT_F32, 1 << 31) == 0
    assert m.dct_select_threshold_workspace_bytes(m.DCT_F32, 1 << 20) > 0
    assert 0 < m.dct_threshold_compact_workspace_bytes(m.DCT_F32, 1 << 28) < (1 << 20)  # O(workgroups), not O(n)
    small = m.dct_select_threshold_workspace_bytes(m.DCT_F32, 1 << 20)
    big = m.dct_select_threshold_workspace_bytes(m.DCT_F32, 1 << 28)
    assert 0 < small < big <= (1 << 28) * 4 // 15  # a candidate buffer of 1/16 of the vector plus a fixed part
    for_k = m.dct_select_threshold_workspace_bytes_for(m.DCT_F32, 1 << 28, 1342178)   # 0.5 % kept
    assert small < for_k < big // 3 and m.dct_select_threshold_workspace_bytes_for(m.DCT_F32, 1 << 28, 0) == 0
    assert m.dct_select_threshold_workspace_bytes_for(m.DCT_F32, 1 << 28, 1 << 27) == big       # half kept: the worst case
    # null pointers and bad sizes are rejected before anything is enqueued
    assert lib.dct_select_threshold(None, 0, 10, 1, None, None, 0, None) == 1
    assert lib.dct_threshold_compact(None, 0, 10, None, 0, None, None, 0, None, None, 0, None) == 1
    assert lib.dct_rowtopk_fwd(None, 0, 1, 1, 1, 1, None, None, None, None) == 1
    assert lib.dct_rowtopk_bwd(None, 0, 1, 1, 1, 1, None, None, None) == 1
    assert "INVALID" in m.dct_status_string(1)


def test_binding_refuses_cpu_tensors():
    import torch
    import paper_2010_08899_amd as m
    g = torch.zeros(16)
    with pytest.raises(ValueError):
        m.dct_select_threshold(g, 1, torch.zeros(4, dtype=torch.int32), torch.zeros(1024, dtype=torch.uint8))


def test_binding_reports_the_error_sentinels():
    """A selection that gave up leaves DCT_TAU_KEY_ERROR in the record, a compaction with a broken
    workspace DCT_COUNT_WORKSPACE_ERROR in the count: the host readers raise on both."""
    import torch
    import paper_2010_08899_amd as m
    header = open(os.path.join(ROOT, "include", "dct.h")).read()
    assert re.search(r"#define\s+DCT_TAU_KEY_ERROR\s+0xFFFFFFFFu", header)
    ok = torch.tensor([0x3F800000, 7, 2, 1], dtype=torch.int32)
    assert tuple(m.read_threshold(ok)) == (0x3F800000, 7, 2, 1)
    with pytest.raises(m.DctError):
        m.read_threshold(torch.tensor([-1, 0, 0, 0], dtype=torch.int32))
    with pytest.raises(m.DctError):
        m.read_count(torch.tensor([-1], dtype=torch.int64))


def test_every_kernel_the_benchmark_prices_has_counter_traffic_on_file():
    """bench.py looks the HBM traffic of its calls up in profiles/hbm_traffic_per_launch.txt by kernel name and
    refuses to run when a name is missing: a renamed kernel must come with fresh counters."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench_for_test", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    table, source = bench.traffic_table()
    assert source.startswith("profiles/hbm_traffic_per_launch.txt#sha1:")
    for call, kernels in bench.CALL_KERNELS.items():
        assert bench.measured_traffic(call, table) > 0, call
        for name, launches in kernels:
            assert name in table and launches >= 1, (call, name)
