"""Host-only checks of the C ABI: the built library loads and exports every entry point that
include/dcpq.h declares, and the Python binding names the same set (no compute calls here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "dcpq.h")
LIB = os.path.join(ROOT, "paper_1905_06900_amd", "libdcpq.so")


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dcpq_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_1905_06900_amd import build
        build.build()
    return ctypes.CDLL(LIB)


def test_header_declares_the_call_list():
    names = declared_symbols()
    for want in ("dcpq_derive_codebooks", "dcpq_build_small_tables", "dcpq_build_tables",
                 "dcpq_scan_candidates", "dcpq_refine_topk", "dcpq_search"):
        assert want in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_symbols():
        assert hasattr(lib, name), name


def test_binding_covers_the_same_symbols():
    from paper_1905_06900_amd import binding
    assert binding.exported_symbols() == declared_symbols()


def test_host_side_queries_need_no_gpu(lib):
    lib.dcpq_version.restype = ctypes.c_int
    assert lib.dcpq_version() >= 1
    lib.dcpq_shape_supported.restype = ctypes.c_int
    assert lib.dcpq_shape_supported(8, 16) == 1 and lib.dcpq_shape_supported(3, 16) == 0
    lib.dcpq_scan_workspace_bytes.restype = ctypes.c_size_t
    lib.dcpq_scan_workspace_bytes.argtypes = [ctypes.c_uint64, ctypes.c_int, ctypes.c_int, ctypes.c_uint32]
    small = lib.dcpq_scan_workspace_bytes(100_000, 8, 16, 1000)
    big = lib.dcpq_scan_workspace_bytes(100_000_000, 8, 4096, 4000)
    assert 0 < small < big
    lib.dcpq_last_error.restype = ctypes.c_char_p
    assert isinstance(lib.dcpq_last_error(), bytes)


def test_scan_plan_covers_every_code_once_and_picks_the_tile_from_the_batch():
    """Host-side planning of the scan: the workgroups of the single pass cover codes 0 .. N without
    overlap, and m = 8 takes the smallest tile that holds the batch."""
    from paper_1905_06900_amd import binding
    for n, nq, r in [(100_000_000, 4096, 4000), (100_000_000, 16, 4000), (5_000_000, 100, 1000), (70_001, 5, 333),
                     (1, 1, 1)]:
        p = binding.scan_plan(n, 8, nq, r)
        assert p["query_tile"] == (16 if nq <= 16 else 32 if nq <= 32 else 64)
        assert p["tiles"] == -(-nq // p["query_tile"])
        assert (p["blocks"] - 1) * p["codes_per_block"] < n <= p["blocks"] * p["codes_per_block"]
        assert 1 <= p["slices"] <= 16 and p["slices"] * p["slice_cap"] >= 10 * r
    forced = binding.scan_plan(100_000_000, 8, 4096, 4000, binding.SCAN_TILE16)
    assert forced["query_tile"] == 16 and forced["tiles"] == 256
    three = binding.scan_plan(70_001, 8, 5, 333, binding.SCAN_THREE_PASS)
    assert three["blocks"] == 0 and three["slices"] == 0
    with pytest.raises(binding.DcpqError):
        binding.scan_plan(1000, 3, 5, 10)


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    from paper_1905_06900_amd import binding
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "missing.so"))
    monkeypatch.setattr(binding, "_lib", None)
    with pytest.raises(FileNotFoundError):
        binding.lib()


def test_search_workspace_covers_a_ragged_last_chunk(lib):
    """The scan lays its scratch out for the batch it is given, and a smaller batch can need more
    (fewer queries: more units, more slices).  The fused search must reserve for the full chunks and
    for the last, ragged one."""
    lib.dcpq_search_workspace_bytes.restype = ctypes.c_size_t
    lib.dcpq_search_workspace_bytes.argtypes = [ctypes.c_uint64, ctypes.c_int, ctypes.c_int, ctypes.c_uint32, ctypes.c_int]
    lib.dcpq_scan_workspace_bytes.restype = ctypes.c_size_t
    lib.dcpq_scan_workspace_bytes.argtypes = [ctypes.c_uint64, ctypes.c_int, ctypes.c_int, ctypes.c_uint32]
    cases = [(10_000_000, 2, 64, 48, 1000), (1000, 1, 32768, 32746, 10), (10_000_000, 16, 8192, 8151, 100),
             (100_000, 8, 64, 1, 500), (5_000_000, 4, 100, 37, 2000)]
    for n, m, chunk, tail, r in cases:
        full_only = lib.dcpq_search_workspace_bytes(n, m, chunk, r, chunk)
        with_tail = lib.dcpq_search_workspace_bytes(n, m, chunk + tail, r, chunk)
        extra = lib.dcpq_scan_workspace_bytes(n, m, tail, r) - lib.dcpq_scan_workspace_bytes(n, m, chunk, r)
        assert with_tail >= full_only
        if extra > 0:
            assert with_tail - full_only >= extra - 256, (n, m, chunk, tail, r)
    # r above the supported range: no size is promised
    assert lib.dcpq_search_workspace_bytes(1 << 28, 8, 16, (1 << 26) + 1, 0) == 0
    assert lib.dcpq_scan_workspace_bytes(1 << 28, 8, 16, (1 << 26) + 1) == 0
