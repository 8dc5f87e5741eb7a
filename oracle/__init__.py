"""CPU oracle for the two-pass derived-codebook PQ search (Alg. 1-3 of the paper).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py``; the GPU library and its Python binding never import it.

The arithmetic lives in ``dcpq_oracle.c`` (plain C, fp32 where an integer is decided, fp64 for
the exact re-ranking).  This module compiles that file with gcc and wraps it with ctypes; it
adds no arithmetic of its own.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dcpq_oracle.c")
_LIB = os.path.join(_HERE, "libdcpq_oracle.so")

# -ffp-contract=off / -fno-fast-math: one IEEE rounding per written fp32 operation.
_CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the C oracle (no-op when the library is newer than the source)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.run(["gcc", *_CFLAGS, _SRC, "-o", tmp, "-lm"], check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.dcpq_oracle_select.restype = C.c_uint64
        _lib.dcpq_oracle_topk.restype = C.c_uint64
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _u16(a):
    return np.ascontiguousarray(a, dtype=np.uint16)


def num_threads() -> int:
    return int(lib().dcpq_oracle_num_threads())


def derive_codebooks(C_full: np.ndarray, b: int = 16, bbar: int = 8) -> np.ndarray:
    """[m][2^b][dsub] -> [m][2^bbar][dsub] (group means by low bbar bits)."""
    C_full = _f32(C_full)
    m, k, dsub = C_full.shape
    assert k == 1 << b
    out = np.empty((m, 1 << bbar, dsub), np.float32)
    lib().dcpq_oracle_derive_codebooks(_p(C_full), m, dsub, b, bbar, _p(out))
    return out


def compute_tables_f32(y: np.ndarray, Cb: np.ndarray) -> np.ndarray:
    Cb = _f32(Cb); y = _f32(y)
    m, kc, dsub = Cb.shape
    assert y.shape == (m * dsub,)
    out = np.empty((m, kc), np.float32)
    lib().dcpq_oracle_compute_tables_f32(_p(y), _p(Cb), m, kc, dsub, _p(out))
    return out


def compute_tables_f64(y: np.ndarray, Cb: np.ndarray) -> np.ndarray:
    Cb = _f32(Cb); y = _f32(y)
    m, kc, dsub = Cb.shape
    assert y.shape == (m * dsub,)
    out = np.empty((m, kc), np.float64)
    lib().dcpq_oracle_compute_tables_f64(_p(y), _p(Cb), m, kc, dsub, _p(out))
    return out


def bounds(Dbar: np.ndarray, codes: np.ndarray, n_first: int, bbar: int = 8):
    Dbar = _f32(Dbar); codes = _u16(codes)
    m = Dbar.shape[0]
    assert Dbar.shape[1] == 1 << bbar and codes.shape[1] == m and n_first <= codes.shape[0]
    lo = C.c_float(); hi = C.c_float()
    lib().dcpq_oracle_bounds(_p(Dbar), m, bbar, _p(codes), C.c_uint64(n_first), C.byref(lo), C.byref(hi))
    return np.float32(lo.value), np.float32(hi.value)


def quantize(Dbar: np.ndarray, qmin, qmax) -> np.ndarray:
    Dbar = _f32(Dbar)
    out = np.empty(Dbar.shape, np.uint8)
    lib().dcpq_oracle_quantize(_p(Dbar), int(Dbar.size), C.c_float(float(qmin)), C.c_float(float(qmax)), _p(out))
    return out


def adc_low_bits(codes: np.ndarray, Qt: np.ndarray, bbar: int = 8) -> np.ndarray:
    codes = _u16(codes); Qt = np.ascontiguousarray(Qt, np.uint8)
    n, m = codes.shape
    assert Qt.shape == (m, 1 << bbar)
    out = np.empty(n, np.uint8)
    lib().dcpq_oracle_adc_low_bits(_p(codes), C.c_uint64(n), m, bbar, _p(Qt), _p(out))
    return out


def select(qd: np.ndarray, r: int, ids: np.ndarray | None = None):
    qd = np.ascontiguousarray(qd, np.uint8)
    n = qd.shape[0]
    if ids is not None:
        ids = np.ascontiguousarray(ids, np.uint32)
    cid = np.empty(r, np.uint32); cqd = np.empty(r, np.uint8)
    kept = lib().dcpq_oracle_select(_p(qd), _p(ids), C.c_uint64(n), C.c_uint64(r), _p(cid), _p(cqd))
    return cid[:kept], cqd[:kept]


def refine(y, C_full, codes, cand_id, b: int = 16) -> np.ndarray:
    y = _f32(y); C_full = _f32(C_full); codes = _u16(codes)
    cand_id = np.ascontiguousarray(cand_id, np.uint32)
    m, k, dsub = C_full.shape
    out = np.empty(cand_id.shape[0], np.float64)
    lib().dcpq_oracle_refine(_p(y), _p(C_full), m, dsub, b, _p(codes), _p(cand_id),
                             C.c_uint64(cand_id.shape[0]), _p(out))
    return out


def topk(dist, ids, k: int):
    dist = np.ascontiguousarray(dist, np.float64); ids = np.ascontiguousarray(ids, np.uint32)
    n = dist.shape[0]
    oi = np.empty(k, np.uint32); od = np.empty(k, np.float64)
    kept = lib().dcpq_oracle_topk(_p(dist), _p(ids), C.c_uint64(n), C.c_uint64(k), _p(oi), _p(od))
    return oi[:kept], od[:kept]


def search_flat(C_full, Cbar, codes, queries, r: int, k: int, b: int = 16, bbar: int = 8) -> dict:
    """Alg. 3 without an index for a batch of queries; returns every intermediate."""
    C_full = _f32(C_full); Cbar = _f32(Cbar); codes = _u16(codes); queries = _f32(queries)
    m, kf, dsub = C_full.shape
    nq = queries.shape[0]; N = codes.shape[0]
    assert kf == 1 << b and Cbar.shape == (m, 1 << bbar, dsub) and queries.shape[1] == m * dsub
    kbar = 1 << bbar
    out = dict(
        small=np.empty((nq, m, kbar), np.float32), bounds=np.empty((nq, 2), np.float32),
        qtab=np.empty((nq, m, kbar), np.uint8), cand_id=np.empty((nq, r), np.uint32),
        cand_qd=np.empty((nq, r), np.uint8), ids=np.empty((nq, k), np.uint32),
        dist=np.empty((nq, k), np.float64))
    rc = lib().dcpq_oracle_search_flat(
        _p(C_full), _p(Cbar), m, dsub, b, bbar, _p(codes), C.c_uint64(N), _p(queries), nq,
        C.c_uint64(r), C.c_uint64(k), _p(out["small"]), _p(out["bounds"]), _p(out["qtab"]),
        _p(out["cand_id"]), _p(out["cand_qd"]), _p(out["ids"]), _p(out["dist"]))
    if rc != 0:
        raise ValueError("dcpq_oracle_search_flat failed: %d" % rc)
    return out


def search_exhaustive(C_full, codes, queries, k: int, b: int = 16):
    """Alg. 1 with full tables over the whole list (what two-pass returns when r = N)."""
    C_full = _f32(C_full); codes = _u16(codes); queries = _f32(queries)
    m, kf, dsub = C_full.shape
    nq = queries.shape[0]; N = codes.shape[0]
    ids = np.empty((nq, k), np.uint32); dist = np.empty((nq, k), np.float64)
    rc = lib().dcpq_oracle_search_exhaustive(_p(C_full), m, dsub, b, _p(codes), C.c_uint64(N),
                                             _p(queries), nq, C.c_uint64(k), _p(ids), _p(dist))
    if rc != 0:
        raise ValueError("dcpq_oracle_search_exhaustive failed: %d" % rc)
    return ids, dist


def ivf_probe(queries, coarse, nprobe: int) -> np.ndarray:
    queries = _f32(queries); coarse = _f32(coarse)
    nq, D = queries.shape; nlist = coarse.shape[0]
    out = np.empty((nq, nprobe), np.int32)
    for q in range(nq):
        lib().dcpq_oracle_ivf_probe(_p(queries[q]), _p(coarse), nlist, D, nprobe, _p(out[q]))
    return out


def search_ivf(C_full, Cbar, codes, offsets, coarse, queries, probe, r: int, k: int,
               b: int = 16, bbar: int = 8) -> dict:
    C_full = _f32(C_full); Cbar = _f32(Cbar); codes = _u16(codes); queries = _f32(queries)
    coarse = _f32(coarse)
    offsets = np.ascontiguousarray(offsets, np.int64); probe = np.ascontiguousarray(probe, np.int32)
    m, kf, dsub = C_full.shape
    nq = queries.shape[0]; nlist = coarse.shape[0]; nprobe = probe.shape[1]
    kbar = 1 << bbar
    assert offsets.shape == (nlist + 1,) and probe.shape[0] == nq
    out = dict(
        bounds=np.empty((nq, 2), np.float32), qtab=np.empty((nq, nprobe, m, kbar), np.uint8),
        cand_id=np.empty((nq, r), np.uint32), cand_qd=np.empty((nq, r), np.uint8),
        count=np.empty(nq, np.uint32), ids=np.empty((nq, k), np.uint32),
        dist=np.empty((nq, k), np.float64))
    rc = lib().dcpq_oracle_search_ivf(
        _p(C_full), _p(Cbar), m, dsub, b, bbar, _p(codes), _p(offsets), _p(coarse), nlist,
        _p(queries), nq, _p(probe), nprobe, C.c_uint64(r), C.c_uint64(k), _p(out["bounds"]),
        _p(out["qtab"]), _p(out["cand_id"]), _p(out["cand_qd"]), _p(out["count"]),
        _p(out["ids"]), _p(out["dist"]))
    if rc != 0:
        raise ValueError("dcpq_oracle_search_ivf failed: %d" % rc)
    return out


# ---- training (Alg. 2) and encoding ---------------------------------------------------------------

def assign(X, Cb, want_dist: bool = False):
    """Nearest centroid of every row of X ([n][d], may be a strided view of a wider array) in Cb ([k][d])."""
    Cb = _f32(Cb)
    X = np.asarray(X, dtype=np.float32)
    assert X.ndim == 2 and X.strides[1] == 4 and X.strides[0] % 4 == 0
    n, d = X.shape
    label = np.empty(n, np.uint32)
    dist = np.empty(n, np.float64) if want_dist else None
    lib().dcpq_oracle_assign(C.c_void_p(X.ctypes.data), C.c_uint64(n), d, X.strides[0] // 4, _p(Cb), Cb.shape[0],
                             _p(label), _p(dist))
    return (label, dist) if want_dist else label


def kmeans(X, C_init, iters: int):
    """Alg. 2 step 1 from given initial centroids -> (centroids [k][d], labels [n])."""
    X = _f32(X); Cb = _f32(C_init).copy()
    n, d = X.shape
    label = np.empty(n, np.uint32)
    lib().dcpq_oracle_kmeans(_p(X), C.c_uint64(n), d, d, Cb.shape[0], iters, _p(Cb), _p(label))
    return Cb, label


def balanced_assign(D):
    """[n][kbar] fp32 distances -> (labels [n] with n / kbar members per cluster, rounds)."""
    D = _f32(D)
    n, kbar = D.shape
    label = np.empty(n, np.uint32)
    rounds = lib().dcpq_oracle_balanced_assign(_p(D), n, kbar, _p(label))
    if rounds < 0:
        raise ValueError("balanced_assign: n must be a positive multiple of kbar")
    return label, rounds


def kmeans_same_size(P, Cbar_init, iters: int):
    """Alg. 2 step 2 -> (centroids [kbar][d] = means of the groups, labels [n])."""
    P = _f32(P); Cbar = _f32(Cbar_init).copy()
    n, d = P.shape
    label = np.empty(n, np.uint32)
    if lib().dcpq_oracle_kmeans_same_size(_p(P), n, d, Cbar.shape[0], iters, _p(Cbar), _p(label)) != 0:
        raise ValueError("kmeans_same_size: bad sizes")
    return Cbar, label


def build_final_codebook(Ct, label, bbar: int):
    """Alg. 2 step 3 -> (final codebook [k][d], perm [k] with perm[final index] = temporary index)."""
    Ct = _f32(Ct); label = np.ascontiguousarray(label, np.uint32)
    k, d = Ct.shape
    Cf = np.empty_like(Ct); perm = np.empty(k, np.uint32)
    if lib().dcpq_oracle_build_final_codebook(_p(Ct), k, d, _p(label), bbar, _p(Cf), _p(perm)) != 0:
        raise ValueError("build_final_codebook: groups are not of equal size")
    return Cf, perm


def encode(X, C_full):
    """[n][m*dsub] vectors -> [n][m] uint16 codes (nearest centroid per sub-vector)."""
    X = _f32(X); C_full = _f32(C_full)
    m, kc, dsub = C_full.shape
    n = X.shape[0]
    assert X.shape[1] == m * dsub
    codes = np.empty((n, m), np.uint16)
    lib().dcpq_oracle_encode(_p(X), C.c_uint64(n), _p(C_full), m, kc, dsub, _p(codes))
    return codes
