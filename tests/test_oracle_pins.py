"""Pins for the CPU oracle: each oracle function is checked against something that is not itself
-- the paper's printed example, closed forms, invariants, textbook reductions and brute force
written independently here (numpy fp64 / python integers / exact rationals)."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny(seed, m=3, dsub=4, b=6, bbar=3, N=400, nq=4, scale=10.0):
    rng = np.random.default_rng(seed)
    C = (rng.normal(size=(m, 1 << b, dsub)) * scale).astype(np.float32)
    codes = rng.integers(0, 1 << b, size=(N, m)).astype(np.uint16)
    queries = (rng.normal(size=(nq, m * dsub)) * scale).astype(np.float32)
    return C, codes, queries


# ------------------------------------------------------------------------------------------------
# low bits / index layout / derive
# ------------------------------------------------------------------------------------------------
def read_golden_example():
    vals = {}
    for line in open(os.path.join(GOLDEN, "fig1c_index_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, *rest = line.split()
        vals[key] = [int(x) for x in rest]
    return vals["b"][0], vals["bbar"][0], vals["cluster"][0], vals["indexes"]


def test_paper_index_example_selects_group_members():
    b, bbar, cluster, indexes = read_golden_example()
    # indicator codebook: 1.0 at the printed indexes, 0 elsewhere -> only that cluster's mean is 1
    C = np.zeros((1, 1 << b, 1), np.float32)
    C[0, indexes, 0] = 1.0
    Cbar = oracle.derive_codebooks(C, b=b, bbar=bbar)
    expect = np.zeros((1, 1 << bbar, 1), np.float32)
    expect[0, cluster, 0] = 1.0
    np.testing.assert_array_equal(Cbar, expect)
    # and the printed indexes are exactly {(i << bbar) | cluster}
    assert sorted(indexes) == [(i << bbar) | cluster for i in range(1 << (b - bbar))]


def test_derive_constant_groups_and_identity():
    rng = np.random.default_rng(0)
    b, bbar, m, dsub = 6, 3, 2, 5
    # dyadic values so that every partial sum is exact in fp32 and the mean is p itself
    p = (rng.integers(-4096, 4096, size=(m, 1 << bbar, dsub)) / 64.0).astype(np.float32)
    C = np.empty((m, 1 << b, dsub), np.float32)
    for i in range(1 << b):
        C[:, i, :] = p[:, i & ((1 << bbar) - 1), :]          # P1: low bits name the group
    np.testing.assert_array_equal(oracle.derive_codebooks(C, b=b, bbar=bbar), p)
    # bbar == b: every group has one member, derived == full
    np.testing.assert_array_equal(oracle.derive_codebooks(C, b=b, bbar=b), C)


def test_derive_matches_fp64_group_mean():
    rng = np.random.default_rng(1)
    b, bbar, m, dsub = 8, 4, 3, 7
    C = (rng.normal(size=(m, 1 << b, dsub)) * 50 + 100).astype(np.float32)
    got = oracle.derive_codebooks(C, b=b, bbar=bbar)
    # group l = rows l, l + 2^bbar, l + 2*2^bbar, ... (stride view, no index formula retyped)
    want = C.astype(np.float64).reshape(m, 1 << (b - bbar), 1 << bbar, dsub).mean(axis=1)
    np.testing.assert_allclose(got, want, rtol=2e-6)
    # high-bits grouping would be a different (wrong) answer on this input
    wrong = C.astype(np.float64).reshape(m, 1 << bbar, 1 << (b - bbar), dsub).mean(axis=2)
    assert np.abs(got - wrong).max() > 1.0


# ------------------------------------------------------------------------------------------------
# Eq. 1 tables
# ------------------------------------------------------------------------------------------------
def test_tables_against_expanded_norm_formula_and_zero_entry():
    C, _, queries = tiny(2, m=3, dsub=5, b=6)
    y = queries[0].copy()
    y[5:10] = C[1, 17]                       # second sub-vector equals centroid 17 of sub-quantizer 1
    got32 = oracle.compute_tables_f32(y, C)
    got64 = oracle.compute_tables_f64(y, C)
    yy = y.astype(np.float64).reshape(3, 1, 5)
    CC = C.astype(np.float64)
    want = (yy ** 2).sum(-1) - 2 * np.einsum("jkt,jkt->jk", np.broadcast_to(yy, CC.shape), CC) + (CC ** 2).sum(-1)
    np.testing.assert_allclose(got64, want, rtol=1e-9, atol=1e-9)
    np.testing.assert_allclose(got32, want, rtol=1e-5, atol=1e-4)
    assert got32[1, 17] == 0.0 and got64[1, 17] == 0.0
    assert (got32 >= 0).all()
    # sub-vector j only meets codebook j: permuting another sub-vector leaves table j unchanged
    y2 = y.copy(); y2[0:5] = y2[0:5][::-1] + 1
    np.testing.assert_array_equal(oracle.compute_tables_f32(y2, C)[1:], got32[1:])
    assert not np.array_equal(oracle.compute_tables_f32(y2, C)[0], got32[0])


def test_tables_f32_is_sequential_single_precision():
    # A sum that differs between fp32-sequential, fp32-pairwise and fp64 orders:
    # (1e8 - 0)^2 ... use values where rounding after each step is visible.
    y = np.array([4097.0, 1.0, 1.0, 1.0], np.float32)       # 4097^2 = 16785409 is not an fp32 number
    C = np.zeros((1, 1, 4), np.float32)
    got = oracle.compute_tables_f32(y, C)[0, 0]
    a = np.float32(4097.0) * np.float32(4097.0)              # rounds to 16785408
    for _ in range(3):
        a = np.float32(a + np.float32(1.0))                  # each +1 is absorbed or rounded in fp32
    assert got == a
    assert oracle.compute_tables_f64(y, C)[0, 0] == 4097.0 ** 2 + 3


# ------------------------------------------------------------------------------------------------
# bounds + quantizer
# ------------------------------------------------------------------------------------------------
def small_adc_py(Dbar, code, bbar):
    """fp32, j increasing -- written with numpy scalars."""
    mask = (1 << bbar) - 1
    acc = np.float32(Dbar[0, int(code[0]) & mask])
    for j in range(1, Dbar.shape[0]):
        acc = np.float32(acc + Dbar[j, int(code[j]) & mask])
    return acc


def test_bounds_invariants():
    C, codes, queries = tiny(3, b=6, bbar=3, N=300)
    Cbar = oracle.derive_codebooks(C, b=6, bbar=3)
    Dbar = oracle.compute_tables_f32(queries[1], Cbar)
    for n_first in (1, 37, 300):
        qmin, qmax = oracle.bounds(Dbar, codes, n_first, bbar=3)
        assert qmin == Dbar.min()
        ds = np.array([small_adc_py(Dbar, codes[i], 3) for i in range(n_first)], np.float32)
        assert qmax == ds.max()
        # only the first n_first codes matter
        tail = codes.copy(); tail[n_first:] = 0
        assert oracle.bounds(Dbar, tail, n_first, bbar=3) == (qmin, qmax)
    # only the low bits of the codes matter
    hi = codes ^ np.uint16(0b111000)
    assert oracle.bounds(Dbar, hi, 300, bbar=3) == oracle.bounds(Dbar, codes, 300, bbar=3)


def test_quantizer_properties_and_exact_rational_check():
    rng = np.random.default_rng(4)
    Dbar = (rng.random((4, 256)) * 1000 + 3).astype(np.float32)
    qmin = np.float32(Dbar.min())
    qmax = np.float32(np.sort(Dbar.ravel())[-40])            # some entries lie above qmax
    Q = oracle.quantize(Dbar, qmin, qmax)
    assert Q.dtype == np.uint8 and Q.shape == Dbar.shape
    assert Q.ravel()[Dbar.argmin()] == 0
    np.testing.assert_array_equal(Q == 255, Dbar >= qmax)      # ">= qmax -> 255", bins 0..254 below
    order = np.argsort(Dbar.ravel(), kind="stable")
    assert (np.diff(Q.ravel()[order].astype(int)) >= 0).all()  # monotone
    # exact rational evaluation of floor((D - qmin) / (qmax - qmin) * 255)
    exact = np.empty(Dbar.size, int)
    for e, d in enumerate(Dbar.ravel()):
        v = (Fraction(float(d)) - Fraction(float(qmin))) / (Fraction(float(qmax)) - Fraction(float(qmin))) * 255
        exact[e] = min(255, v.numerator // v.denominator)
    diff = Q.ravel().astype(int) - exact
    assert np.abs(diff).max() <= 1                              # fp32 rounding can move an edge case by one bin
    assert (diff != 0).mean() < 0.01
    # floor, not round-to-nearest: the mid-bin value stays in its bin
    mid = np.array([[np.float32(qmin + (qmax - qmin) * (10.7 / 255.0))]], np.float32)
    assert oracle.quantize(mid, qmin, qmax)[0, 0] == 10


def test_quantizer_degenerate_range():
    Dbar = np.full((2, 8), 5.0, np.float32)
    assert (oracle.quantize(Dbar, 5.0, 5.0) == 0).all()
    assert (oracle.quantize(Dbar, 5.0, 4.0) == 0).all()


def test_first_r_codes_never_exceed_bucket_255_before_saturation():
    # Floor property: for a code among the first r, sum_j Q_j <= 255 (d - m*qmin)/(qmax-qmin) <= 255
    C, codes, queries = tiny(5, m=4, b=8, bbar=4, N=500)
    Cbar = oracle.derive_codebooks(C, b=8, bbar=4)
    for y in queries:
        Dbar = oracle.compute_tables_f32(y, Cbar)
        qmin, qmax = oracle.bounds(Dbar, codes, 200, bbar=4)
        Q = oracle.quantize(Dbar, qmin, qmax).astype(int)
        low = codes[:200] & 15
        sums = sum(Q[j, low[:, j]] for j in range(4))
        assert sums.max() <= 255 + 1      # +1: a single entry equal to qmax is clamped up to 255


# ------------------------------------------------------------------------------------------------
# scan / select
# ------------------------------------------------------------------------------------------------
def test_adc_low_bits_bruteforce_and_saturation():
    rng = np.random.default_rng(6)
    m, bbar, N = 5, 3, 200
    Qt = rng.integers(0, 100, size=(m, 1 << bbar)).astype(np.uint8)   # sums straddle 255
    codes = rng.integers(0, 1 << 16, size=(N, m)).astype(np.uint16)
    got = oracle.adc_low_bits(codes, Qt, bbar=bbar)
    want = [min(255, sum(int(Qt[j, int(codes[i, j]) % (1 << bbar)]) for j in range(m))) for i in range(N)]
    np.testing.assert_array_equal(got, np.array(want, np.uint8))
    assert (got == 255).any() and (got < 255).any()
    # high bits are ignored
    np.testing.assert_array_equal(oracle.adc_low_bits(codes | np.uint16(0xFF00), Qt, bbar=bbar), got)


@pytest.mark.parametrize("r", [1, 7, 50, 333])
def test_select_is_r_smallest_by_qd_then_id(r):
    rng = np.random.default_rng(7)
    qd = rng.integers(0, 9, size=333).astype(np.uint8)       # many ties
    cid, cqd = oracle.select(qd, r)
    want = sorted(range(333), key=lambda i: (int(qd[i]), i))[:r]
    np.testing.assert_array_equal(cid, np.array(want, np.uint32))
    np.testing.assert_array_equal(cqd, qd[want])
    if r == 333:
        assert sorted(cid.tolist()) == list(range(333))


def test_select_with_id_map():
    qd = np.array([3, 1, 3, 1, 0], np.uint8)
    ids = np.array([10, 20, 30, 40, 50], np.uint32)
    cid, cqd = oracle.select(qd, 4, ids)
    assert cid.tolist() == [50, 20, 40, 10] and cqd.tolist() == [0, 1, 1, 3]


# ------------------------------------------------------------------------------------------------
# refine / top-k / whole search
# ------------------------------------------------------------------------------------------------
def decode_np(C, codes):
    return np.concatenate([C[j][codes[:, j].astype(int)] for j in range(C.shape[0])], axis=1).astype(np.float64)


def test_refine_equals_distance_to_decoded_vector():
    C, codes, queries = tiny(8, m=4, dsub=6, b=7, N=150)
    cand = np.array([3, 149, 0, 77, 77], np.uint32)
    got = oracle.refine(queries[2], C, codes, cand, b=7)
    want = ((queries[2].astype(np.float64)[None, :] - decode_np(C, codes[cand])) ** 2).sum(1)
    np.testing.assert_allclose(got, want, rtol=1e-12)
    # Eq. 2 == Eq. 3: gather from the fp64 tables and add
    T = oracle.compute_tables_f64(queries[2], C)
    via_tables = np.array([sum(T[j, codes[i, j]] for j in range(4)) for i in cand])
    np.testing.assert_allclose(got, via_tables, rtol=1e-12)


def test_topk_sorted_by_distance_then_id():
    d = np.array([5.0, 1.0, 5.0, 0.5, 1.0, 9.0])
    ids = np.array([60, 50, 40, 30, 20, 10], np.uint32)
    oi, od = oracle.topk(d, ids, 4)
    assert oi.tolist() == [30, 20, 50, 40] and od.tolist() == [0.5, 1.0, 1.0, 5.0]
    oi, _ = oracle.topk(d, ids, 6)
    assert oi.tolist() == [30, 20, 50, 40, 60, 10]


def exhaustive_np(C, codes, queries, k):
    X = decode_np(C, codes)
    out = []
    for y in queries.astype(np.float64):
        d = ((X - y[None, :]) ** 2).sum(1)
        order = np.lexsort((np.arange(len(d)), d))[:k]
        out.append(order)
    return np.array(out, np.uint32)


def test_exhaustive_search_matches_numpy_bruteforce():
    C, codes, queries = tiny(9, m=3, dsub=4, b=6, N=300, nq=5)
    ids, dist = oracle.search_exhaustive(C, codes, queries, 10, b=6)
    np.testing.assert_array_equal(ids, exhaustive_np(C, codes, queries, 10))
    assert (np.diff(dist, axis=1) >= 0).all()


def test_exhaustive_search_of_an_8_bit_quantizer_matches_numpy_bruteforce():
    # the "plain 8-bit" comparison system: PQ 8x8, every sub-code below 256
    C, codes, queries = tiny(19, m=8, dsub=2, b=8, N=700, nq=4)
    assert codes.max() < 256 and C.shape == (8, 256, 2)
    ids, dist = oracle.search_exhaustive(C, codes, queries, 25, b=8)
    np.testing.assert_array_equal(ids, exhaustive_np(C, codes, queries, 25))
    X = decode_np(C, codes)
    for q in range(4):
        want = ((X[ids[q]] - queries[q].astype(np.float64)[None, :]) ** 2).sum(1)
        np.testing.assert_allclose(dist[q], want, rtol=1e-12)


def test_two_pass_with_r_equal_N_is_exhaustive_adc():
    C, codes, queries = tiny(10, m=3, dsub=4, b=6, bbar=3, N=300, nq=6)
    Cbar = oracle.derive_codebooks(C, b=6, bbar=3)
    out = oracle.search_flat(C, Cbar, codes, queries, r=300, k=12, b=6, bbar=3)
    ids, dist = oracle.search_exhaustive(C, codes, queries, 12, b=6)
    np.testing.assert_array_equal(out["ids"], ids)
    np.testing.assert_allclose(out["dist"], dist, rtol=1e-12)
    for q in range(6):
        assert sorted(out["cand_id"][q].tolist()) == list(range(300))


def test_two_pass_result_is_exact_topk_of_candidate_set_and_intermediates_compose():
    C, codes, queries = tiny(11, m=4, dsub=3, b=8, bbar=4, N=2000, nq=5)
    Cbar = oracle.derive_codebooks(C, b=8, bbar=4)
    r, k = 150, 20
    out = oracle.search_flat(C, Cbar, codes, queries, r=r, k=k, b=8, bbar=4)
    X = decode_np(C, codes)
    for q in range(5):
        y = queries[q]
        Dbar = oracle.compute_tables_f32(y, Cbar)
        np.testing.assert_array_equal(out["small"][q], Dbar)
        qmin, qmax = oracle.bounds(Dbar, codes, r, bbar=4)
        assert tuple(out["bounds"][q]) == (qmin, qmax)
        Qt = oracle.quantize(Dbar, qmin, qmax)
        np.testing.assert_array_equal(out["qtab"][q], Qt)
        qd = oracle.adc_low_bits(codes, Qt, bbar=4)
        want = sorted(range(2000), key=lambda i: (int(qd[i]), i))[:r]
        np.testing.assert_array_equal(out["cand_id"][q], np.array(want, np.uint32))
        np.testing.assert_array_equal(out["cand_qd"][q], qd[want])
        cand = np.array(want)
        d = ((X[cand] - y.astype(np.float64)[None, :]) ** 2).sum(1)
        order = np.lexsort((cand, d))[:k]
        np.testing.assert_array_equal(out["ids"][q], cand[order].astype(np.uint32))
        np.testing.assert_allclose(out["dist"][q], d[order], rtol=1e-12)


def test_hierarchical_codebooks_make_pass_one_useful():
    """Statistical sanity (not parity): with parents in the low bits the candidate set of a modest
    r holds nearly all of the exact top-k -- the paper's own criterion for choosing r2 (Sec. 4.2)."""
    import torch
    from paper_1905_06900_amd import synth
    w = synth.scaled(synth.WORKLOADS[0], N=20000, Q=8, r=1000)
    d = synth.make_flat(w, "cpu")
    C = d["codebooks"].numpy(); codes = synth.to_numpy(d["codes"]); queries = d["queries"].numpy()
    Cbar = oracle.derive_codebooks(C)
    out = oracle.search_flat(C, Cbar, codes, queries, r=w.r, k=20)
    ids, _ = oracle.search_exhaustive(C, codes, queries, 20)
    overlap = np.mean([len(set(out["ids"][q]) & set(ids[q])) / 20 for q in range(8)])
    assert overlap >= 0.9


# ------------------------------------------------------------------------------------------------
# inverted index variant
# ------------------------------------------------------------------------------------------------
def tiny_ivf(seed, nlist=6, m=3, dsub=4, b=6, N=500, nq=4):
    rng = np.random.default_rng(seed)
    C, codes, queries = tiny(seed, m=m, dsub=dsub, b=b, N=N, nq=nq)
    coarse = (rng.normal(size=(nlist, m * dsub)) * 10).astype(np.float32)
    cuts = np.sort(rng.integers(0, N + 1, size=nlist - 1))
    offsets = np.concatenate([[0], cuts, [N]]).astype(np.int64)
    return C, codes, queries, coarse, offsets


def test_ivf_probe_bruteforce():
    C, codes, queries, coarse, offsets = tiny_ivf(12)
    probe = oracle.ivf_probe(queries, coarse, 3)
    for q in range(len(queries)):
        d = ((coarse.astype(np.float64) - queries[q].astype(np.float64)[None, :]) ** 2).sum(1)
        np.testing.assert_array_equal(probe[q], np.lexsort((np.arange(len(d)), d))[:3])


def test_ivf_with_zero_centres_and_all_lists_probed_is_the_flat_search():
    C, codes, queries, coarse, offsets = tiny_ivf(13)
    coarse[:] = 0.0
    Cbar = oracle.derive_codebooks(C, b=6, bbar=3)
    nlist = coarse.shape[0]
    probe = np.tile(np.arange(nlist, dtype=np.int32), (len(queries), 1))   # probe order == id order
    iv = oracle.search_ivf(C, Cbar, codes, offsets, coarse, queries, probe, r=60, k=10, b=6, bbar=3)
    fl = oracle.search_flat(C, Cbar, codes, queries, r=60, k=10, b=6, bbar=3)
    np.testing.assert_array_equal(iv["bounds"], fl["bounds"])
    np.testing.assert_array_equal(iv["cand_id"], fl["cand_id"])
    np.testing.assert_array_equal(iv["cand_qd"], fl["cand_qd"])
    np.testing.assert_array_equal(iv["ids"], fl["ids"])
    np.testing.assert_allclose(iv["dist"], fl["dist"], rtol=1e-12)
    for p in range(nlist):
        np.testing.assert_array_equal(iv["qtab"][:, p], fl["qtab"])
    assert (iv["count"] == 60).all()


def test_ivf_residual_search_against_bruteforce_on_reconstructions():
    C, codes, queries, coarse, offsets = tiny_ivf(14, nlist=8, N=800)
    Cbar = oracle.derive_codebooks(C, b=6, bbar=3)
    nprobe, r, k = 3, 40, 8
    probe = oracle.ivf_probe(queries, coarse, nprobe)
    iv = oracle.search_ivf(C, Cbar, codes, offsets, coarse, queries, probe, r=r, k=k, b=6, bbar=3)
    list_of = np.searchsorted(offsets, np.arange(800), side="right") - 1
    recon = decode_np(C, codes) + coarse.astype(np.float64)[list_of]      # x ~ c_l + pq(residual)
    for q in range(len(queries)):
        y = queries[q]
        in_probed = np.isin(list_of, probe[q])
        total = int(in_probed.sum())
        ncand = min(r, total)
        assert iv["count"][q] == ncand
        cand = iv["cand_id"][q][:ncand].astype(int)
        assert in_probed[cand].all()
        # pass one recomputed with per-list residual tables and the per-query bounds
        qmin, qmax = iv["bounds"][q]
        tabs = {}
        lo = np.inf
        for p, l in enumerate(probe[q]):
            rho = (y - coarse[l]).astype(np.float32)
            tabs[l] = oracle.compute_tables_f32(rho, Cbar)
            lo = min(lo, tabs[l].min())
        assert qmin == np.float32(lo)
        walk = [i for l in probe[q] for i in range(offsets[l], offsets[l + 1])][:r]
        hi = max(small_adc_py(tabs[list_of[i]], codes[i], 3) for i in walk)
        assert qmax == hi
        qd = np.full(800, 999)
        for p, l in enumerate(probe[q]):
            Qt = oracle.quantize(tabs[l], qmin, qmax)
            np.testing.assert_array_equal(iv["qtab"][q, p], Qt)
            sl = slice(offsets[l], offsets[l + 1])
            qd[sl] = oracle.adc_low_bits(codes[sl], Qt, bbar=3)
        want = sorted(np.nonzero(in_probed)[0], key=lambda i: (qd[i], i))[:r]
        np.testing.assert_array_equal(cand, want)
        # pass two: exact distance to the reconstruction, top-k by (d, id)
        d = ((recon[cand] - y.astype(np.float64)[None, :]) ** 2).sum(1)
        order = np.lexsort((cand, d))[:k]
        kk = min(k, ncand)
        np.testing.assert_array_equal(iv["ids"][q][:kk], cand[order][:kk])
        np.testing.assert_allclose(iv["dist"][q][:kk], d[order][:kk], rtol=1e-9)


def test_ivf_pads_when_probed_lists_are_short():
    C, codes, queries, coarse, offsets = tiny_ivf(15, nlist=5, N=100)
    offsets = np.array([0, 2, 2, 5, 50, 100], np.int64)
    Cbar = oracle.derive_codebooks(C, b=6, bbar=3)
    probe = np.tile(np.array([[1, 0, 2]], np.int32), (len(queries), 1))     # 0 + 2 + 3 = 5 codes
    iv = oracle.search_ivf(C, Cbar, codes, offsets, coarse, queries, probe, r=8, k=6, b=6, bbar=3)
    assert (iv["count"] == 5).all()
    assert (iv["cand_id"][:, 5:] == 0xFFFFFFFF).all() and (iv["cand_qd"][:, 5:] == 255).all()
    assert (iv["ids"][:, 5:] == 0xFFFFFFFF).all() and np.isinf(iv["dist"][:, 5:]).all()
    assert (np.sort(iv["cand_id"][:, :5], axis=1) == np.arange(5)).all()
