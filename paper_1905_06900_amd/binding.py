"""Thin Python binding of libdcpq (see include/dcpq.h): argument marshalling only.

torch supplies device memory and the current HIP stream; every step of the search runs inside
the library's kernels.  Functions carry the names of the C entry points without the prefix.
There is no CPU fallback: if the library has not been built, importing symbols from it raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libdcpq.so")

OK, EINVAL, EWORKSPACE, EHIP, EUNSUPPORTED = 0, 1, 2, 3, 4
PAD_ID = 0xFFFFFFFF


class DcpqError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("dcpq error %d: %s" % (code, msg))
        self.code = code


_lib = None

_vp, _i, _u32, _u64, _sz = C.c_void_p, C.c_int, C.c_uint32, C.c_uint64, C.c_size_t

_SIGNATURES = {
    "dcpq_last_error": (C.c_char_p, []),
    "dcpq_version": (_i, []),
    "dcpq_shape_supported": (_i, [_i, _i]),
    "dcpq_derive_codebooks": (_i, [_vp, _i, _i, _vp, _vp]),
    "dcpq_build_small_tables": (_i, [_vp, _i, _vp, _i, _i, _vp, _u64, _u32, _vp, _vp, _vp, _vp]),
    "dcpq_bits_supported": (_i, [_i, _i]),
    "dcpq_derive_codebooks_bits": (_i, [_vp, _i, _i, _i, _i, _vp, _vp]),
    "dcpq_build_small_tables_bits": (_i, [_vp, _i, _vp, _i, _i, _i, _vp, _i, _u64, _u32, _vp, _vp, _vp, _vp]),
    "dcpq_refine_topk_bits": (_i, [_vp, _u32, _vp, _i, _u64, _i, _vp, _i, _u32, _u32, _vp, _vp, _vp, _sz, _vp]),
    "dcpq_search_bits_chunk": (_i, [_i, _i, _i, _i]),
    "dcpq_search_bits_workspace_bytes": (_sz, [_u64, _i, _i, _u32, _i, _i]),
    "dcpq_search_bits": (_i, [_vp, _i, _vp, _vp, _i, _i, _i, _i, _vp, _u64, _u32, _u32, _i, _vp, _vp, _i, _vp, _sz, _vp]),
    "dcpq_search_refine_mode": (_i, [_i, _i, _i, _i, _u32, _i]),
    "dcpq_refine_direct_topk": (_i, [_vp, _vp, _i, _i, _i, _vp, _u64, _vp, _i, _u32, _u32, _vp, _vp, _vp, _sz, _vp]),
    "dcpq_assign": (_i, [_vp, _u64, _i, _vp, _i, _i, _i, _vp, _i, _vp, _vp]),
    "dcpq_encode": (_i, [_vp, _u64, _vp, _i, _i, _i, _vp, _vp]),
    "dcpq_kmeans_workspace_bytes": (_sz, [_i, _i]),
    "dcpq_kmeans": (_i, [_vp, _u64, _i, _i, _i, _i, _vp, _vp, _vp, _sz, _vp]),
    "dcpq_kmeans_same_size_workspace_bytes": (_sz, [_i, _i, _i]),
    "dcpq_kmeans_same_size": (_i, [_vp, _i, _i, _i, _i, _vp, _vp, _vp, _sz, _vp]),
    "dcpq_build_final_codebook": (_i, [_vp, _i, _i, _vp, _i, _vp, _vp, _vp]),
    "dcpq_build_quantizers_workspace_bytes": (_sz, [_u64, _i, _i, _i]),
    "dcpq_build_quantizers": (_i, [_vp, _u64, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, _sz, _vp]),
    "dcpq_build_tables": (_i, [_vp, _i, _vp, _i, _i, _vp, _vp]),
    "dcpq_build_tables_n": (_i, [_vp, _i, _vp, _i, _i, _i, _vp, _vp]),
    "dcpq_plain_workspace_bytes": (_sz, [_u64, _i, _u32]),
    "dcpq_plain_search": (_i, [_vp, _u32, _vp, _i, _u64, _i, _i, _u32, _vp, _vp, _vp, _sz, _vp]),
    "dcpq_scan_workspace_bytes": (_sz, [_u64, _i, _i, _u32]),
    "dcpq_scan_candidates": (_i, [_vp, _u64, _i, _vp, _i, _u32, _vp, _vp, _vp, _sz, _vp]),
    "dcpq_scan_query_tile": (_i, [_i]),
    "dcpq_scan_plan": (_i, [_u64, _i, _i, _u32, _i, _vp, _i]),
    "dcpq_search_chunk": (_i, [_i, _i, _i]),
    "dcpq_scan_candidates_mode": (_i, [_vp, _u64, _i, _vp, _i, _u32, _vp, _vp, _vp, _sz, _i, _vp]),
    "dcpq_scan_candidates_packed": (_i, [_vp, _u64, _i, _vp, _i, _u32, _vp, _vp, _vp, _sz, _i, _vp]),
    "dcpq_static_scratch_bytes": (_sz, []),
    "dcpq_scan_candidates_static": (_i, [_vp, _u64, _i, _vp, _i, _u32, _vp, _vp, _vp]),
    "dcpq_refine_workspace_bytes": (_sz, [_i, _u32]),
    "dcpq_refine_topk": (_i, [_vp, _vp, _u64, _i, _vp, _i, _u32, _u32, _vp, _vp, _vp, _sz, _vp]),
    "dcpq_search_workspace_bytes": (_sz, [_u64, _i, _i, _u32, _i]),
    "dcpq_ivf_probe_workspace_bytes": (_sz, [_i, _i]),
    "dcpq_ivf_probe": (_i, [_vp, _i, _i, _vp, _i, _i, _vp, _vp, _sz, _vp]),
    "dcpq_ivf_tables_workspace_bytes": (_sz, [_i]),
    "dcpq_ivf_tables_workspace_bytes_fast": (_sz, [_i, _i, _i]),
    "dcpq_ivf_build_small_tables": (_i, [_vp, _i, _vp, _i, _vp, _i, _vp, _i, _i, _vp, _vp, _u32, _vp, _vp, _vp, _sz, _vp]),
    "dcpq_ivf_scan_workspace_bytes": (_sz, [_i, _u32]),
    "dcpq_ivf_scan_candidates": (_i, [_vp, _vp, _i, _i, _vp, _i, _vp, _i, _u32, _vp, _vp, _vp, _vp, _sz, _vp]),
    "dcpq_ivf_scan_candidates_packed": (_i, [_vp, _vp, _i, _i, _vp, _i, _vp, _i, _u32, _vp, _vp, _vp, _vp, _sz, _vp]),
    "dcpq_pack_low_bytes": (_i, [_vp, _u64, _i, _vp, _vp]),
    "dcpq_ivf_refine_workspace_bytes": (_sz, [_i, _u32]),
    "dcpq_ivf_refine_topk": (_i, [_vp, _vp, _i, _vp, _i, _i, _vp, _vp, _vp, _i, _vp, _i, _u32, _u32, _vp, _vp, _vp, _sz, _vp]),
    "dcpq_ivf_search_workspace_bytes": (_sz, [_i, _i, _i, _i, _u32]),
    "dcpq_ivf_search": (_i, [_vp, _i, _vp, _i, _i, _vp, _vp, _i, _i, _vp, _vp, _vp, _u32, _u32, _vp, _vp, _vp, _sz, _vp]),
    "dcpq_profile_enable": (_i, [_i]),
    "dcpq_profile_stage_count": (_i, []),
    "dcpq_profile_stage_name": (C.c_char_p, [_i]),
    "dcpq_profile_read": (_i, [_i, C.POINTER(C.c_double), C.POINTER(C.c_uint64)]),
    "dcpq_profile_copy": (_i, [_vp, _vp, _sz, _vp]),
    "dcpq_profile_stream_read_sink_bytes": (_sz, []),
    "dcpq_profile_stream_read": (_i, [_vp, _sz, _vp, _vp]),
    "dcpq_search": (_i, [_vp, _i, _vp, _vp, _i, _i, _vp, _u64, _u32, _u32, _vp, _vp, _i, _vp, _sz, _vp]),
}


def exported_symbols() -> list[str]:
    return sorted(_SIGNATURES)


def lib() -> C.CDLL:
    """Loads the built library; raises if it is missing (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                "%s not built: run `python -m paper_1905_06900_amd.build` (hipcc, gfx950)" % LIB_PATH)
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            f = getattr(l, name)
            f.restype = res
            f.argtypes = args
        _lib = l
    return _lib


def _check(rc: int):
    if rc != OK:
        raise DcpqError(rc, lib().dcpq_last_error().decode())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, dtype, name: str) -> int:
    if not (t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise TypeError("%s must be a contiguous %s tensor on the GPU" % (name, dtype))
    return t.data_ptr()


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def version() -> int:
    return int(lib().dcpq_version())


def _bits_of(n_entries: int) -> int:
    b = n_entries.bit_length() - 1
    assert 1 << b == n_entries, "table / codebook sizes are powers of two"
    return b


def derive_codebooks(codebooks: torch.Tensor, bbar: int = 8) -> torch.Tensor:
    """Sec. 3.2: [m][2^b][dsub] -> [m][2^bbar][dsub], the means of the centroids sharing their low bbar bits"""
    m, k, dsub = codebooks.shape
    b = _bits_of(k)
    out = torch.empty((m, 1 << bbar, dsub), dtype=torch.float32, device=codebooks.device)
    if (b, bbar) == (16, 8):
        _check(lib().dcpq_derive_codebooks(_dev(codebooks, torch.float32, "codebooks"), m, dsub,
                                           out.data_ptr(), _stream()))
    else:
        _check(lib().dcpq_derive_codebooks_bits(_dev(codebooks, torch.float32, "codebooks"), m, dsub, b, bbar,
                                                out.data_ptr(), _stream()))
    return out


def build_small_tables(queries: torch.Tensor, derived: torch.Tensor, codes: torch.Tensor, r: int,
                       want_small: bool = False):
    """-> (qtab u8 [nq][m][256], bounds f32 [nq][2], small f32 [nq][m][2^bbar] or None); bbar from `derived`,
    the sub-code width from the dtype of `codes` (uint16 or uint8)"""
    m, ks, dsub = derived.shape
    bbar = _bits_of(ks)
    nq = queries.shape[0]
    assert queries.shape[1] == m * dsub and codes.shape[1] == m
    dev = queries.device
    qtab = torch.empty((nq, m, 256), dtype=torch.uint8, device=dev)
    bounds = torch.empty((nq, 2), dtype=torch.float32, device=dev)
    small = torch.empty((nq, m, ks), dtype=torch.float32, device=dev) if want_small else None
    if bbar == 8 and codes.dtype == torch.uint16:
        _check(lib().dcpq_build_small_tables(
            _dev(queries, torch.float32, "queries"), nq, _dev(derived, torch.float32, "derived"), m, dsub,
            _dev(codes, torch.uint16, "codes"), codes.shape[0], r, qtab.data_ptr(), bounds.data_ptr(),
            small.data_ptr() if small is not None else None, _stream()))
    else:
        assert codes.dtype in (torch.uint8, torch.uint16)
        _check(lib().dcpq_build_small_tables_bits(
            _dev(queries, torch.float32, "queries"), nq, _dev(derived, torch.float32, "derived"), m, dsub, bbar,
            _dev(codes, codes.dtype, "codes"), codes.element_size(), codes.shape[0], r, qtab.data_ptr(),
            bounds.data_ptr(), small.data_ptr() if small is not None else None, _stream()))
    return qtab, bounds, small


def build_tables(queries: torch.Tensor, codebooks: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    m, k, dsub = codebooks.shape
    nq = queries.shape[0]
    assert k == 65536 and queries.shape[1] == m * dsub
    if out is None:
        out = torch.empty((nq, m, 65536), dtype=torch.float32, device=queries.device)
    _check(lib().dcpq_build_tables(_dev(queries, torch.float32, "queries"), nq,
                                   _dev(codebooks, torch.float32, "codebooks"), m, dsub,
                                   _dev(out, torch.float32, "tables"), _stream()))
    return out


def build_tables_n(queries: torch.Tensor, codebooks: torch.Tensor) -> torch.Tensor:
    """Eq. 1 for codebooks of any size: [nq][D] x [m][n_entries][dsub] -> [nq][m][n_entries] fp32"""
    m, n_entries, dsub = codebooks.shape
    nq = queries.shape[0]
    assert queries.shape[1] == m * dsub
    tables = torch.empty((nq, m, n_entries), dtype=torch.float32, device=queries.device)
    _check(lib().dcpq_build_tables_n(_dev(queries, torch.float32, "queries"), nq, _dev(codebooks, torch.float32, "codebooks"),
                                     m, dsub, n_entries, tables.data_ptr(), _stream()))
    return tables


def plain_workspace_bytes(n: int, nq: int, k: int) -> int:
    return lib().dcpq_plain_workspace_bytes(n, nq, k)


def plain_search(tables: torch.Tensor, codes: torch.Tensor, k: int, workspace: torch.Tensor | None = None):
    """Alg. 1 with full floating-point tables over every code -> (ids u32 [nq][k], dist f32 [nq][k])"""
    nq, m, n_entries = tables.shape
    n = codes.shape[0]
    assert codes.shape[1] == m and codes.dtype in (torch.uint8, torch.uint16)
    dev = tables.device
    ids = torch.empty((nq, k), dtype=torch.uint32, device=dev)
    dist = torch.empty((nq, k), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = _workspace(lib().dcpq_plain_workspace_bytes(n, nq, k), dev)
    _check(lib().dcpq_plain_search(_dev(tables, torch.float32, "tables"), n_entries, _dev(codes, codes.dtype, "codes"),
                                   codes.element_size(), n, m, nq, k, ids.data_ptr(), dist.data_ptr(),
                                   workspace.data_ptr(), workspace.numel(), _stream()))
    return ids, dist


def scan_workspace_bytes(n_codes: int, m: int, nq: int, r: int) -> int:
    return int(lib().dcpq_scan_workspace_bytes(n_codes, m, nq, r))


def scan_query_tile(m: int) -> int:
    return int(lib().dcpq_scan_query_tile(m))


def search_chunk(m: int, nq: int, chunk_queries: int = 0) -> int:
    return int(lib().dcpq_search_chunk(m, nq, chunk_queries))


SCAN_AUTO, SCAN_THREE_PASS, SCAN_TILE16, SCAN_TILE32, SCAN_TILE64 = 0, 1, 2, 3, 4


def scan_plan(n_codes: int, m: int, nq: int, r: int, mode: int = SCAN_AUTO) -> dict:
    """How the scan lays out its work for this problem (see dcpq_scan_plan)."""
    info = (C.c_uint64 * 10)()
    _check(lib().dcpq_scan_plan(n_codes, m, nq, r, mode, C.cast(info, C.c_void_p), 10))
    keys = ("query_tile", "tiles", "blocks", "codes_per_block", "slices", "slice_cap", "sample_runs", "sample_stride",
            "pilot_every", "pilot_rank")
    return dict(zip(keys, (int(v) for v in info)))


def scan_candidates(codes: torch.Tensor, qtab: torch.Tensor, r: int, workspace: torch.Tensor | None = None,
                    mode: int = SCAN_AUTO):
    """-> (cand_id u32 [nq][r], cand_qd u8 [nq][r]) sorted by (qd, id)"""
    n, m = codes.shape
    nq = qtab.shape[0]
    assert qtab.shape[1:] == (m, 256)
    dev = codes.device
    cand_id = torch.empty((nq, r), dtype=torch.uint32, device=dev)
    cand_qd = torch.empty((nq, r), dtype=torch.uint8, device=dev)
    if workspace is None:
        workspace = _workspace(scan_workspace_bytes(n, m, nq, r), dev)
    if codes.dtype == torch.uint8:          # the low-byte plane of the codes
        _check(lib().dcpq_scan_candidates_packed(_dev(codes, torch.uint8, "plane"), n, m, _dev(qtab, torch.uint8, "qtab"),
                                                 nq, r, cand_id.data_ptr(), cand_qd.data_ptr(), workspace.data_ptr(),
                                                 workspace.numel(), mode, _stream()))
        return cand_id, cand_qd
    if mode == SCAN_AUTO:
        _check(lib().dcpq_scan_candidates(_dev(codes, torch.uint16, "codes"), n, m, _dev(qtab, torch.uint8, "qtab"),
                                          nq, r, cand_id.data_ptr(), cand_qd.data_ptr(), workspace.data_ptr(),
                                          workspace.numel(), _stream()))
    else:
        _check(lib().dcpq_scan_candidates_mode(_dev(codes, torch.uint16, "codes"), n, m,
                                               _dev(qtab, torch.uint8, "qtab"), nq, r, cand_id.data_ptr(),
                                               cand_qd.data_ptr(), workspace.data_ptr(), workspace.numel(), mode,
                                               _stream()))
    return cand_id, cand_qd


def scan_candidates_static(codes: torch.Tensor, qtab: torch.Tensor, r: int, cand_id: torch.Tensor,
                           cand_qd: torch.Tensor):
    """The scan through the entry point that allocates nothing: outputs are the caller's tensors,
    the scratch memory is the library's static array (dcpq_static_scratch_bytes())."""
    n, m = codes.shape
    nq = qtab.shape[0]
    assert qtab.shape[1:] == (m, 256) and cand_id.shape == (nq, r) and cand_qd.shape == (nq, r)
    _check(lib().dcpq_scan_candidates_static(_dev(codes, torch.uint16, "codes"), n, m, _dev(qtab, torch.uint8, "qtab"),
                                             nq, r, _dev(cand_id, torch.uint32, "cand_id"),
                                             _dev(cand_qd, torch.uint8, "cand_qd"), _stream()))
    return cand_id, cand_qd


def refine_topk(tables: torch.Tensor, codes: torch.Tensor, cand_id: torch.Tensor, k: int,
                workspace: torch.Tensor | None = None):
    """-> (ids u32 [nq][k], dist f32 [nq][k]) ascending by (dist, id); tables [nq][m][2^b], codes uint16 (b = 16)
    or uint8 (b = 8)"""
    n, m = codes.shape
    nq, r = cand_id.shape
    n_entries = tables.shape[2]
    assert tables.shape == (nq, m, n_entries)
    dev = codes.device
    ids = torch.empty((nq, k), dtype=torch.uint32, device=dev)
    dist = torch.empty((nq, k), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = _workspace(lib().dcpq_refine_workspace_bytes(nq, r), dev)
    if n_entries == 65536 and codes.dtype == torch.uint16:
        _check(lib().dcpq_refine_topk(_dev(tables, torch.float32, "tables"), _dev(codes, torch.uint16, "codes"), n, m,
                                      _dev(cand_id, torch.uint32, "cand_id"), nq, r, k, ids.data_ptr(),
                                      dist.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream()))
    else:
        assert codes.dtype in (torch.uint8, torch.uint16)
        _check(lib().dcpq_refine_topk_bits(_dev(tables, torch.float32, "tables"), n_entries, _dev(codes, codes.dtype, "codes"),
                                           codes.element_size(), n, m, _dev(cand_id, torch.uint32, "cand_id"), nq, r, k,
                                           ids.data_ptr(), dist.data_ptr(), workspace.data_ptr(), workspace.numel(),
                                           _stream()))
    return ids, dist


REFINE_AUTO, REFINE_TABLES, REFINE_DIRECT, REFINE_SPLIT = 0, 1, 2, 3


def search_refine_mode(m: int, dsub: int, b: int, nq: int, r: int, refine_mode: int = REFINE_AUTO) -> int:
    """The mode pass two of `search` runs in for (the first chunk of) a batch of nq queries."""
    return int(lib().dcpq_search_refine_mode(m, dsub, b, nq, r, refine_mode))


def refine_direct_topk(queries: torch.Tensor, codebooks: torch.Tensor, codes: torch.Tensor, cand_id: torch.Tensor,
                       k: int, workspace: torch.Tensor | None = None):
    """Pass two with table entries computed on demand -> (ids u32 [nq][k], dist f32 [nq][k])"""
    n, m = codes.shape
    nq, r = cand_id.shape
    _, kf, dsub = codebooks.shape
    b = _bits_of(kf)
    assert codes.element_size() * 8 == b and queries.shape == (nq, m * dsub)
    dev = codes.device
    ids = torch.empty((nq, k), dtype=torch.uint32, device=dev)
    dist = torch.empty((nq, k), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = _workspace(lib().dcpq_refine_workspace_bytes(nq, r), dev)
    _check(lib().dcpq_refine_direct_topk(_dev(queries, torch.float32, "queries"), _dev(codebooks, torch.float32, "codebooks"),
                                         m, dsub, b, _dev(codes, codes.dtype, "codes"), n,
                                         _dev(cand_id, torch.uint32, "cand_id"), nq, r, k, ids.data_ptr(), dist.data_ptr(),
                                         workspace.data_ptr(), workspace.numel(), _stream()))
    return ids, dist


def search_workspace_bytes(n_codes: int, m: int, nq: int, r: int, chunk_queries: int = 0, b: int = 16) -> int:
    if b == 16:
        return int(lib().dcpq_search_workspace_bytes(n_codes, m, nq, r, chunk_queries))
    return int(lib().dcpq_search_bits_workspace_bytes(n_codes, m, nq, r, b, chunk_queries))


def search(queries: torch.Tensor, codebooks: torch.Tensor, derived: torch.Tensor, codes: torch.Tensor,
           r: int, k: int, chunk_queries: int = 0, workspace: torch.Tensor | None = None,
           ids: torch.Tensor | None = None, dist: torch.Tensor | None = None, refine_mode: int = REFINE_AUTO):
    """Alg. 3 end to end without an index -> (ids u32 [nq][k], dist f32 [nq][k]); b from `codebooks`
    ([m][2^b][dsub]), bbar from `derived` ([m][2^bbar][dsub])"""
    m, kf, dsub = codebooks.shape
    b, bbar = _bits_of(kf), _bits_of(derived.shape[1])
    n = codes.shape[0]
    nq = queries.shape[0]
    assert queries.shape[1] == m * dsub and codes.shape[1] == m and derived.shape == (m, 1 << bbar, dsub)
    assert codes.element_size() * 8 == b, "sub-codes of b bits are stored in b / 8 bytes"
    dev = queries.device
    if ids is None:
        ids = torch.empty((nq, k), dtype=torch.uint32, device=dev)
    if dist is None:
        dist = torch.empty((nq, k), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = _workspace(search_workspace_bytes(n, m, nq, r, chunk_queries, b), dev)
    if (b, bbar) == (16, 8) and refine_mode == REFINE_AUTO:
        _check(lib().dcpq_search(_dev(queries, torch.float32, "queries"), nq,
                                 _dev(codebooks, torch.float32, "codebooks"), _dev(derived, torch.float32, "derived"),
                                 m, dsub, _dev(codes, torch.uint16, "codes"), n, r, k, ids.data_ptr(), dist.data_ptr(),
                                 chunk_queries, workspace.data_ptr(), workspace.numel(), _stream()))
    else:
        _check(lib().dcpq_search_bits(_dev(queries, torch.float32, "queries"), nq,
                                      _dev(codebooks, torch.float32, "codebooks"), _dev(derived, torch.float32, "derived"),
                                      m, dsub, b, bbar, _dev(codes, codes.dtype, "codes"), n, r, k, refine_mode,
                                      ids.data_ptr(), dist.data_ptr(), chunk_queries, workspace.data_ptr(), workspace.numel(), _stream()))
    return ids, dist


# ---- training and encoding (Alg. 2) ------------------------------------------------------------

def assign(points: torch.Tensor, codebooks: torch.Tensor, want_dist: bool = False, label_dtype=torch.int32):
    """Nearest centroid per sub-vector: points [n][m*dsub], codebooks [m][n_entries][dsub] -> labels [n][m]"""
    m, ne, dsub = codebooks.shape
    n = points.shape[0]
    assert points.shape[1] == m * dsub
    labels = torch.empty((n, m), dtype=label_dtype, device=points.device)
    dist = torch.empty((n, m), dtype=torch.float32, device=points.device) if want_dist else None
    _check(lib().dcpq_assign(_dev(points, torch.float32, "points"), n, m * dsub, _dev(codebooks, torch.float32, "codebooks"),
                             m, dsub, ne, labels.data_ptr(), labels.element_size(),
                             dist.data_ptr() if dist is not None else None, _stream()))
    return (labels, dist) if want_dist else labels


def encode(vectors: torch.Tensor, codebooks: torch.Tensor) -> torch.Tensor:
    """[n][m*dsub] vectors -> [n][m] codes (uint16 for 2^16 centroids, uint8 for 2^8)"""
    m, kf, dsub = codebooks.shape
    b = _bits_of(kf)
    n = vectors.shape[0]
    codes = torch.empty((n, m), dtype=torch.uint16 if b == 16 else torch.uint8, device=vectors.device)
    _check(lib().dcpq_encode(_dev(vectors, torch.float32, "vectors"), n, _dev(codebooks, torch.float32, "codebooks"),
                             m, dsub, b, codes.data_ptr(), _stream()))
    return codes


def kmeans(points: torch.Tensor, init: torch.Tensor, iters: int):
    """Alg. 2 step 1 from given initial centroids -> (centroids [k][d], labels int32 [n])"""
    n, d = points.shape
    k = init.shape[0]
    cent = init.clone()
    labels = torch.empty(n, dtype=torch.int32, device=points.device)
    ws = _workspace(lib().dcpq_kmeans_workspace_bytes(k, d), points.device)
    _check(lib().dcpq_kmeans(_dev(points, torch.float32, "points"), n, d, d, k, iters, _dev(cent, torch.float32, "centroids"),
                             labels.data_ptr(), ws.data_ptr(), ws.numel(), _stream()))
    return cent, labels


def kmeans_same_size(points: torch.Tensor, init: torch.Tensor, iters: int):
    """Alg. 2 step 2 -> (centroids [kbar][d] = means of the groups, labels int32 [n]); synchronizes"""
    n, d = points.shape
    kbar = init.shape[0]
    cent = init.clone()
    labels = torch.empty(n, dtype=torch.int32, device=points.device)
    ws = _workspace(lib().dcpq_kmeans_same_size_workspace_bytes(n, d, kbar), points.device)
    _check(lib().dcpq_kmeans_same_size(_dev(points, torch.float32, "points"), n, d, kbar, iters,
                                       _dev(cent, torch.float32, "centroids"), labels.data_ptr(), ws.data_ptr(), ws.numel(),
                                       _stream()))
    return cent, labels


def build_final_codebook(temp: torch.Tensor, labels: torch.Tensor, bbar: int):
    """Alg. 2 step 3 -> (final codebook [k][d], perm int32 [k], perm[final index] = temporary index)"""
    k, d = temp.shape
    final = torch.empty_like(temp)
    perm = torch.empty(k, dtype=torch.int32, device=temp.device)
    _check(lib().dcpq_build_final_codebook(_dev(temp, torch.float32, "temp"), k, d, _dev(labels, torch.int32, "labels"), bbar,
                                           final.data_ptr(), perm.data_ptr(), _stream()))
    return final, perm


def build_quantizers(train: torch.Tensor, init_codebooks: torch.Tensor, bbar: int, iters: int, iters_same_size: int):
    """All of Alg. 2: train [n][m*dsub], init_codebooks [m][2^b][dsub] -> (codebooks, derived [m][2^bbar][dsub])"""
    m, kf, dsub = init_codebooks.shape
    b = _bits_of(kf)
    n = train.shape[0]
    cb = init_codebooks.clone()
    derived = torch.empty((m, 1 << bbar, dsub), dtype=torch.float32, device=train.device)
    ws = _workspace(lib().dcpq_build_quantizers_workspace_bytes(n, dsub, b, bbar), train.device)
    _check(lib().dcpq_build_quantizers(_dev(train, torch.float32, "train"), n, m, dsub, b, bbar, iters, iters_same_size,
                                       _dev(cb, torch.float32, "codebooks"), derived.data_ptr(), ws.data_ptr(), ws.numel(),
                                       _stream()))
    return cb, derived


def stream_read_gbs(t: torch.Tensor, reps: int = 3) -> float:
    """GB/s of the read-only stream kernel over the bytes of `t` (timed with torch events on the current stream)."""
    nbytes = t.numel() * t.element_size() // 16 * 16
    sink = torch.empty(lib().dcpq_profile_stream_read_sink_bytes(), dtype=torch.uint8, device=t.device)
    _check(lib().dcpq_profile_stream_read(t.data_ptr(), nbytes, sink.data_ptr(), _stream()))
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        _check(lib().dcpq_profile_stream_read(t.data_ptr(), nbytes, sink.data_ptr(), _stream()))
    b.record()
    b.synchronize()
    return nbytes * reps / (a.elapsed_time(b) * 1e-3) / 1e9


def profile_enable(on: bool) -> None:
    _check(lib().dcpq_profile_enable(1 if on else 0))


def profile_read() -> dict:
    """{stage name: (total milliseconds, launches)} since profile_enable(True)."""
    out = {}
    l = lib()
    for s in range(l.dcpq_profile_stage_count()):
        ms, n = C.c_double(), C.c_uint64()
        _check(l.dcpq_profile_read(s, C.byref(ms), C.byref(n)))
        out[l.dcpq_profile_stage_name(s).decode()] = (ms.value, int(n.value))
    return out


# ---- inverted-index variant ---------------------------------------------------------------------
def ivf_probe(queries: torch.Tensor, coarse: torch.Tensor, nprobe: int) -> torch.Tensor:
    """-> probe int32 [nq][nprobe], ordered by (distance, list id)"""
    nq, D = queries.shape
    nlist = coarse.shape[0]
    assert coarse.shape[1] == D
    dev = queries.device
    probe = torch.empty((nq, nprobe), dtype=torch.int32, device=dev)
    ws = _workspace(lib().dcpq_ivf_probe_workspace_bytes(nq, nlist), dev)
    _check(lib().dcpq_ivf_probe(_dev(queries, torch.float32, "queries"), nq, D, _dev(coarse, torch.float32, "coarse"),
                                nlist, nprobe, probe.data_ptr(), ws.data_ptr(), ws.numel(), _stream()))
    return probe


def ivf_build_small_tables(queries, coarse, probe, derived, codes, offsets, r: int, keep_entries: bool = False):
    """-> (qtab u8 [nq][nprobe][m][256], bounds f32 [nq][2]); keep_entries: give the call the workspace with which
    it keeps the table entries between its two passes instead of computing them twice (same results)"""
    m, _, dsub = derived.shape
    nq, nprobe = probe.shape
    nlist = coarse.shape[0]
    assert queries.shape == (nq, m * dsub) and coarse.shape[1] == m * dsub and codes.shape[1] == m
    dev = queries.device
    qtab = torch.empty((nq, nprobe, m, 256), dtype=torch.uint8, device=dev)
    bounds = torch.empty((nq, 2), dtype=torch.float32, device=dev)
    ws = _workspace(lib().dcpq_ivf_tables_workspace_bytes_fast(nq, nprobe, m) if keep_entries
                    else lib().dcpq_ivf_tables_workspace_bytes(nq), dev)
    _check(lib().dcpq_ivf_build_small_tables(
        _dev(queries, torch.float32, "queries"), nq, _dev(coarse, torch.float32, "coarse"), nlist,
        _dev(probe, torch.int32, "probe"), nprobe, _dev(derived, torch.float32, "derived"), m, dsub,
        _dev(codes, torch.uint16, "codes"), _dev(offsets, torch.int64, "offsets"), r, qtab.data_ptr(),
        bounds.data_ptr(), ws.data_ptr(), ws.numel(), _stream()))
    return qtab, bounds


def pack_low_bytes(codes: torch.Tensor) -> torch.Tensor:
    """-> plane u8 [n][m], plane[i][j] = codes[i][j] & 255"""
    n, m = codes.shape
    plane = torch.empty((n, m), dtype=torch.uint8, device=codes.device)
    _check(lib().dcpq_pack_low_bytes(_dev(codes, torch.uint16, "codes"), n, m, plane.data_ptr(), _stream()))
    return plane


def ivf_scan_candidates(codes, offsets, probe, qtab, r: int):
    """-> (cand_id u32 [nq][r], cand_qd u8 [nq][r], count u32 [nq]); codes: the u16 codes or their u8 low-byte plane"""
    m = codes.shape[1]
    nq, nprobe = probe.shape
    nlist = offsets.shape[0] - 1
    dev = codes.device
    cand_id = torch.empty((nq, r), dtype=torch.uint32, device=dev)
    cand_qd = torch.empty((nq, r), dtype=torch.uint8, device=dev)
    count = torch.empty((nq,), dtype=torch.uint32, device=dev)
    ws = _workspace(lib().dcpq_ivf_scan_workspace_bytes(nq, r), dev)
    packed = codes.dtype == torch.uint8
    fn = lib().dcpq_ivf_scan_candidates_packed if packed else lib().dcpq_ivf_scan_candidates
    _check(fn(
        _dev(codes, torch.uint8 if packed else torch.uint16, "codes"), _dev(offsets, torch.int64, "offsets"), nlist, m,
        _dev(probe, torch.int32, "probe"), nprobe, _dev(qtab, torch.uint8, "qtab"), nq, r, cand_id.data_ptr(),
        cand_qd.data_ptr(), count.data_ptr(), ws.data_ptr(), ws.numel(), _stream()))
    return cand_id, cand_qd, count


def ivf_refine_topk(queries, coarse, codebooks, codes, offsets, probe, cand_id, k: int):
    """-> (ids u32 [nq][k], dist f32 [nq][k])"""
    m, _, dsub = codebooks.shape
    nq, r = cand_id.shape
    nprobe = probe.shape[1]
    nlist = coarse.shape[0]
    assert queries.shape == (nq, m * dsub) and coarse.shape[1] == m * dsub and codes.shape[1] == m
    assert probe.shape[0] == nq
    dev = queries.device
    ids = torch.empty((nq, k), dtype=torch.uint32, device=dev)
    dist = torch.empty((nq, k), dtype=torch.float32, device=dev)
    ws = _workspace(lib().dcpq_ivf_refine_workspace_bytes(nq, r), dev)
    _check(lib().dcpq_ivf_refine_topk(
        _dev(queries, torch.float32, "queries"), _dev(coarse, torch.float32, "coarse"), nlist,
        _dev(codebooks, torch.float32, "codebooks"), m, dsub, _dev(codes, torch.uint16, "codes"),
        _dev(offsets, torch.int64, "offsets"), _dev(probe, torch.int32, "probe"), nprobe,
        _dev(cand_id, torch.uint32, "cand_id"), nq, r, k, ids.data_ptr(), dist.data_ptr(), ws.data_ptr(),
        ws.numel(), _stream()))
    return ids, dist


def ivf_search_workspace_bytes(nq: int, nlist: int, nprobe: int, m: int, r: int) -> int:
    return lib().dcpq_ivf_search_workspace_bytes(nq, nlist, nprobe, m, r)


def ivf_search(queries, coarse, codebooks, derived, codes, offsets, nprobe: int, r: int, k: int, plane=None,
               workspace=None, ids=None, dist=None):
    """Index, Tables, Scan, Refine in one call -> (ids u32 [nq][k], dist f32 [nq][k])"""
    m, _, dsub = codebooks.shape
    nq = queries.shape[0]
    nlist = coarse.shape[0]
    assert queries.shape == (nq, m * dsub) and coarse.shape[1] == m * dsub and codes.shape[1] == m
    dev = queries.device
    if ids is None:
        ids = torch.empty((nq, k), dtype=torch.uint32, device=dev)
    if dist is None:
        dist = torch.empty((nq, k), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = _workspace(ivf_search_workspace_bytes(nq, nlist, nprobe, m, r), dev)
    _check(lib().dcpq_ivf_search(
        _dev(queries, torch.float32, "queries"), nq, _dev(coarse, torch.float32, "coarse"), nlist, nprobe,
        _dev(codebooks, torch.float32, "codebooks"), _dev(derived, torch.float32, "derived"), m, dsub,
        _dev(codes, torch.uint16, "codes"), 0 if plane is None else _dev(plane, torch.uint8, "plane"),
        _dev(offsets, torch.int64, "offsets"), r, k, ids.data_ptr(), dist.data_ptr(), workspace.data_ptr(),
        workspace.numel(), _stream()))
    return ids, dist


def profile_copy(src: torch.Tensor, dst: torch.Tensor) -> None:
    """Calibration copy kernel of known size (for scaling hardware traffic counters)."""
    assert src.numel() * src.element_size() == dst.numel() * dst.element_size()
    _check(lib().dcpq_profile_copy(src.data_ptr(), dst.data_ptr(), src.numel() * src.element_size(), _stream()))
