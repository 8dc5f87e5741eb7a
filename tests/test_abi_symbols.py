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


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    from paper_1905_06900_amd import binding
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "missing.so"))
    monkeypatch.setattr(binding, "_lib", None)
    with pytest.raises(FileNotFoundError):
        binding.lib()
