"""GPU parity tests of the flat (no index) path, stage by stage, through the C ABI.

Sizes: the oracle finishes each case in seconds, while N spans many scan units, several query
tiles and ragged tails (N not a multiple of 64, Q not a multiple of the query tile)."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from paper_1905_06900_amd import binding, synth
from parity import FlatCase, to_np, assert_topk_matches, REL_TOL

pytestmark = pytest.mark.gpu

DEV = "cuda"


def small_flat(cfg, N, Q, r, **kw):
    return synth.scaled(synth.WORKLOADS[cfg], N=N, Q=Q, r=r, **kw)


@pytest.fixture(scope="module")
def case0():
    print("case0: cfg0 recipe N=200003 Q=37 r=1000", flush=True)
    return FlatCase(small_flat(0, 200_003, 37, 1000), DEV).run_stages().oracle()


def test_cfg0_scaled_pass_one_bit_exact(case0):
    case0.check_pass_one()


def test_cfg0_scaled_pass_two(case0):
    case0.check_pass_two()


def test_cfg0_scaled_fused_search_matches_staged(case0):
    c = case0
    ids, dist = binding.search(c.queries, c.cb, c.derived, c.codes, c.w.r, c.w.k, chunk_queries=16,
                               refine_mode=binding.REFINE_TABLES)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_np(ids), to_np(c.ids))
    np.testing.assert_array_equal(to_np(dist), to_np(c.dist))


def test_cfg0_scaled_on_demand_refinement(case0):
    # pass two with table entries computed on demand: staged and fused agree bit for bit, both match the
    # oracle, and the default mode of the fused search is this one for the shape (r <= 2^16 / 8)
    c = case0
    assert binding.search_refine_mode(c.w.m, c.w.dsub, 16, c.w.Q, c.w.r) == binding.REFINE_DIRECT
    assert binding.search_refine_mode(c.w.m, c.w.dsub, 16, c.w.Q, 10_000) == binding.REFINE_TABLES
    sids, sdist = binding.refine_direct_topk(c.queries, c.cb, c.codes, c.cand_id, c.w.k)
    fids, fdist = binding.search(c.queries, c.cb, c.derived, c.codes, c.w.r, c.w.k, chunk_queries=16)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_np(fids), to_np(sids))
    np.testing.assert_array_equal(to_np(fdist), to_np(sdist))
    c.check_pass_two(sids, sdist)
    # against the table mode: the same distances up to the last bit
    np.testing.assert_allclose(to_np(sdist), to_np(c.dist), rtol=2e-7)


@pytest.mark.parametrize("cfg,N,Q,r,chunk", [(0, 90_001, 37, 1000, 16), (2, 150_001, 290, 4000, 280),
                                             (4, 40_001, 21, 700, 0)])
def test_split_on_demand_refinement(cfg, N, Q, r, chunk):
    # Pass two split by sub-quantizer (m = 4: two parts of the candidates per sub-quantizer; m = 8: one
    # sub-quantizer per slice; m = 16: two) gives the bits of the one-kernel form, with a ragged last chunk too,
    # and matches the oracle.  The middle case is large enough for the library to pick the split form by itself
    # for the full chunk (280 x 4000 candidates) and the one-kernel form for the last 10 queries.
    w = small_flat(cfg, N, Q, r)
    print("split refinement: cfg%d recipe N=%d Q=%d r=%d chunk=%d" % (cfg, N, Q, r, chunk), flush=True)
    c = FlatCase(w, DEV)
    dids, ddist = binding.search(c.queries, c.cb, c.derived, c.codes, r, w.k, chunk_queries=chunk,
                                 refine_mode=binding.REFINE_DIRECT)
    sids, sdist = binding.search(c.queries, c.cb, c.derived, c.codes, r, w.k, chunk_queries=chunk,
                                 refine_mode=binding.REFINE_SPLIT)
    aids, adist = binding.search(c.queries, c.cb, c.derived, c.codes, r, w.k, chunk_queries=chunk)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_np(sids), to_np(dids))
    np.testing.assert_array_equal(to_np(sdist), to_np(ddist))
    np.testing.assert_array_equal(to_np(aids), to_np(dids))
    np.testing.assert_array_equal(to_np(adist), to_np(ddist))
    if cfg == 2:
        assert binding.search_refine_mode(w.m, w.dsub, 16, 280, r) == binding.REFINE_SPLIT
        assert binding.search_refine_mode(w.m, w.dsub, 16, 10, r) == binding.REFINE_DIRECT
    c.oracle(qsel=np.arange(0, Q, max(1, Q // 24)))
    c.check_pass_two(sids, sdist)


def test_on_demand_refinement_with_r_above_the_lds_sort():
    # r = 9000 candidates per query: the refinement's keys go to the global spill area instead of LDS (and the default
    # mode would be full tables); the on-demand forms, memoized (tie-heavy cfg0 codes repeat sub-codes) and split,
    # still agree bit for bit and with the oracle
    w = small_flat(0, 100_003, 5, 9000)
    print("on-demand refinement, keys spilled: m=%d N=%d Q=%d r=%d" % (w.m, w.N, w.Q, w.r), flush=True)
    c = FlatCase(w, DEV)
    assert binding.search_refine_mode(w.m, w.dsub, 16, w.Q, w.r) == binding.REFINE_TABLES
    dids, ddist = binding.search(c.queries, c.cb, c.derived, c.codes, w.r, w.k, refine_mode=binding.REFINE_DIRECT)
    sids, sdist = binding.search(c.queries, c.cb, c.derived, c.codes, w.r, w.k, refine_mode=binding.REFINE_SPLIT)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_np(dids), to_np(sids))
    np.testing.assert_array_equal(to_np(ddist), to_np(sdist))
    c.oracle()
    c.check_pass_two(dids, ddist)


@pytest.mark.parametrize("case", ["few distinct sub-codes", "set too small"])
def test_on_demand_refinement_with_memoized_entries(case):
    # The one-kernel on-demand refinement collects the distinct (sub-quantizer, sub-code) pairs of a query's
    # candidates in a hash set and computes each entry once (it does so from r m >= 8192 on).  First case: encoded
    # data, where a few dozen sub-codes repeat and the set is used.  Second case: 600 different sub-codes per
    # sub-quantizer (m = 4: 512 slots each): sub-codes do repeat, but the sets cannot hold them, and the kernel falls
    # back to computing per candidate.  Either way: the bits of the split form (which never memoizes), and the
    # oracle's results.
    if case == "few distinct sub-codes":
        w = small_flat(4, 40_001, 21, 1100)                       # GIST-like recipe, m = 16: 17600 pairs per query
        c = FlatCase(w, DEV)
    else:
        w = dataclasses.replace(small_flat(0, 100_003, 9, 4200), data="custom")
        g = torch.Generator(device=DEV); g.manual_seed(991)
        cb = synth.hierarchical_codebooks(w.m, w.dsub, w.b, w.pbits, lambda shape, gg: 40.0 * torch.rand(
            shape, generator=gg, device=DEV, dtype=torch.float32), 4.0, DEV, 992)
        values = torch.randperm(65536, generator=g, device=DEV)[:600]
        codes = values[torch.randint(0, 600, (w.N, w.m), generator=g, device=DEV)].to(torch.int32).to(torch.int16).view(torch.uint16)
        queries = 40.0 * torch.rand((w.Q, w.m * w.dsub), generator=g, device=DEV, dtype=torch.float32)
        c = FlatCase(w, DEV, data=dict(codebooks=cb, codes=codes, queries=queries))
    print("memoized refinement, %s: m=%d N=%d Q=%d r=%d" % (case, w.m, w.N, w.Q, w.r), flush=True)
    dids, ddist = binding.search(c.queries, c.cb, c.derived, c.codes, w.r, w.k, refine_mode=binding.REFINE_DIRECT)
    sids, sdist = binding.search(c.queries, c.cb, c.derived, c.codes, w.r, w.k, refine_mode=binding.REFINE_SPLIT)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_np(dids), to_np(sids))
    np.testing.assert_array_equal(to_np(ddist), to_np(sdist))
    c.oracle()
    c.check_pass_two(dids, ddist)


def test_memoized_refinement_that_gives_up_late_or_meets_padding():
    # Candidate lists written by hand for the stand-alone refinement call.  Query 0: the first candidates repeat 20
    # sub-codes per sub-quantizer (the first collecting pass finds repetition and goes on), the later ones are all
    # different (the sets fill up after that check: entries per candidate after all).  Query 1: only repeating
    # candidates (the memoized form runs to the end), with unused slots (id 0xFFFFFFFF) scattered through the list
    # and at its end.  Query 2: the first 256 all different (given up at the first check).  Each against the oracle's Eq. 3 distances and top-k.
    m, dsub, N, r, k = 8, 16, 6000, 5000, 50
    g = torch.Generator(device=DEV); g.manual_seed(4711)
    cb = 30.0 * torch.rand((m, 65536, dsub), generator=g, device=DEV, dtype=torch.float32)
    few = torch.randint(0, 65536, (20, m), generator=g, device=DEV)
    codes = torch.randint(0, 65536, (N, m), generator=g, device=DEV)
    pick = torch.randint(0, 20, (2000, m), generator=g, device=DEV)
    codes[:2000] = torch.gather(few, 0, pick)
    codes = codes.to(torch.int32).to(torch.int16).view(torch.uint16)
    queries = 30.0 * torch.rand((3, m * dsub), generator=g, device=DEV, dtype=torch.float32)
    cand = torch.full((3, r), 0xFFFFFFFF, dtype=torch.int64, device=DEV)
    cand[0] = torch.arange(r, device=DEV)                                  # 2000 repeating, then 3000 different
    cand[1, :3800:2] = torch.randperm(2000, generator=g, device=DEV)[:1900]   # repeating ones, every other slot unused
    perm = 1000 + torch.randperm(5000, generator=g, device=DEV)
    cand[2] = torch.cat([2000 + torch.arange(256, device=DEV), perm[(perm < 2000) | (perm >= 2256)]])   # nothing repeats at first
    cand_id = cand.to(torch.uint32)
    print("memoized refinement on hand-made candidate lists: m=%d N=%d r=%d" % (m, N, r), flush=True)
    ids, dist = binding.refine_direct_topk(queries, cb, codes, cand_id, k)
    torch.cuda.synchronize()
    ids, dist = to_np(ids), to_np(dist)
    cb_np, codes_np, q_np, cand_np = to_np(cb), to_np(codes), to_np(queries), to_np(cand_id)
    for q in range(3):
        real = cand_np[q][cand_np[q] != 0xFFFFFFFF]
        exact = oracle.refine(q_np[q], cb_np, codes_np, real)
        ref_ids, ref_dist = oracle.topk(exact, real, k)
        assert_topk_matches(ids[q], dist[q], ref_ids, ref_dist, oracle.refine(q_np[q], cb_np, codes_np, ids[q]),
                            cand_ref=real, tag="query %d" % q)


def test_fused_search_m2_with_a_ragged_last_chunk():
    # m = 2 goes through the three-pass scan, whose scratch layout depends on the batch size: the
    # last chunk (48 queries after a chunk of 64) lays it out differently from the full chunks
    w = dataclasses.replace(small_flat(2, 120_007, 112, 300), m=2, dsub=12)
    print("fused search m=2 N=%d Q=%d chunk 64" % (w.N, w.Q), flush=True)
    dev = DEV
    cb = synth.hierarchical_codebooks(2, 12, w.b, w.pbits, lambda shape, g: 0.3 * torch.randn(
        shape, generator=g, device=dev, dtype=torch.float32), 0.03, dev, w.seed + 1)
    codes = synth.random_codes(w.N, 2, dev, w.seed + 2).view(torch.uint16)
    g = torch.Generator(device=dev); g.manual_seed(w.seed + 3)
    queries = 0.3 * torch.randn((w.Q, 24), generator=g, device=dev, dtype=torch.float32)
    c = FlatCase(w, dev, data=dict(codebooks=cb, codes=codes, queries=queries))
    ids, dist = binding.search(c.queries, c.cb, c.derived, c.codes, w.r, w.k, chunk_queries=64)
    torch.cuda.synchronize()
    c.oracle(qsel=[0, 63, 64, 65, 100, 111])
    c.check_pass_two(ids, dist)


def test_full_tables_against_fp64_definition(case0):
    c = case0
    T = to_np(c.tables)
    for q in (0, 17, 36):
        want = oracle.compute_tables_f64(c.q_np[q], c.cb_np)
        np.testing.assert_allclose(T[q], want, rtol=1e-6, atol=1e-30)


@pytest.mark.parametrize("cfg,N,Q,r", [(2, 150_001, 21, 700), (4, 60_000, 9, 5000)])
def test_random_code_recipes_scaled(cfg, N, Q, r):
    # cfg 2's own recipe (random codes, Deep-like queries) and cfg 4's shape (m=16, dsub=60) with
    # random codes instead of the encoded ones (encoding is exercised in the full-size test).
    print("case: cfg%d N=%d Q=%d r=%d" % (cfg, N, Q, r), flush=True)
    w = small_flat(cfg, N, Q, r)
    if cfg == 4:
        w = dataclasses.replace(w, data="deep_random_codes")
        data = synth.make_flat(w, DEV)
        # GIST-like queries and codebook scale for the 960-d shape
        g = synth.WORKLOADS[4]
        data["codebooks"] = synth.hierarchical_codebooks(g.m, g.dsub, 16, 4, synth._uniform(0.0, 0.3, DEV), 0.03, DEV, 5)
        data["queries"] = synth.gist_like(Q, DEV, 6, 7).contiguous()
        c = FlatCase(w, DEV, data)
    else:
        c = FlatCase(w, DEV)
    c.run_stages().oracle()
    c.check_pass_one()
    c.check_pass_two()


def test_sift_recipe_scaled_with_encoded_codes():
    print("case: cfg1 recipe N=30000 Q=19 r=500 (nearest-centroid encoded)", flush=True)
    c = FlatCase(small_flat(1, 30_000, 19, 500), DEV).run_stages().oracle()
    c.check_pass_one()
    c.check_pass_two()


# ------------------------------------------------------------------------------------------------
# edge cases of the scan / select
# ------------------------------------------------------------------------------------------------
def scan_vs_oracle(codes_np, qtab_np, r, modes=(binding.SCAN_AUTO, binding.SCAN_THREE_PASS)):
    """Both scan algorithms (single pass with redo, and three-pass) against the oracle."""
    codes = torch.from_numpy(codes_np.view(np.int16)).to(DEV).view(torch.uint16)
    qtab = torch.from_numpy(qtab_np).to(DEV)
    want = []
    for q in range(qtab_np.shape[0]):
        qd = oracle.adc_low_bits(codes_np, qtab_np[q])
        want.append(oracle.select(qd, r))
    # the codes as stored, and their low-byte plane (the only bytes pass one consumes): same candidates
    plane = binding.pack_low_bytes(codes)
    for src, what in ((codes, "codes"), (plane, "plane")):
        for mode in modes:
            cid, cqd = binding.scan_candidates(src, qtab, r, mode=mode)
            torch.cuda.synchronize()
            cid, cqd = to_np(cid), to_np(cqd)
            for q, (wid, wqd) in enumerate(want):
                np.testing.assert_array_equal(cid[q], wid, err_msg="%s mode %d query %d ids" % (what, mode, q))
                np.testing.assert_array_equal(cqd[q], wqd, err_msg="%s mode %d query %d qd" % (what, mode, q))


@pytest.mark.parametrize("m", [1, 2, 4, 8, 16, 32])
def test_scan_every_supported_m(m):
    rng = np.random.default_rng(m)
    N, Q, r = 70_001, 5, 333
    codes = rng.integers(0, 65536, size=(N, m)).astype(np.uint16)
    qtab = rng.integers(0, 256 // m + 8, size=(Q, m, 256)).astype(np.uint8)
    print("scan m=%d N=%d" % (m, N), flush=True)
    scan_vs_oracle(codes, qtab, r)


@pytest.mark.parametrize("Q", [1, 16, 17, 37, 70])
def test_scan_every_query_tile_size(Q):
    """m = 8 has single-pass kernels for tiles of 16, 32 and 64 queries (the smaller tiles keep repeated
    copies of the tables in LDS); each must give the oracle's candidates for full, ragged and absent
    tiles.  AUTO picks the tile from the batch size."""
    rng = np.random.default_rng(1000 + Q)
    N, r = 90_003, 500
    codes = rng.integers(0, 65536, size=(N, 8)).astype(np.uint16)
    qtab = rng.integers(0, 40, size=(Q, 8, 256)).astype(np.uint8)
    print("scan tiles Q=%d" % Q, flush=True)
    scan_vs_oracle(codes, qtab, r, modes=(binding.SCAN_TILE16, binding.SCAN_TILE32, binding.SCAN_TILE64,
                                          binding.SCAN_AUTO))


@pytest.mark.parametrize("N,r", [(1, 1), (63, 63), (64, 1), (65, 65), (1000, 1000), (5000, 4097), (20000, 9000)])
def test_scan_tiny_and_r_equal_n(N, r):
    rng = np.random.default_rng(N)
    codes = rng.integers(0, 65536, size=(N, 8)).astype(np.uint16)
    qtab = rng.integers(0, 40, size=(3, 8, 256)).astype(np.uint8)
    print("scan N=%d r=%d" % (N, r), flush=True)
    scan_vs_oracle(codes, qtab, r)


def test_scan_giant_ties_and_saturation():
    rng = np.random.default_rng(99)
    N, r = 100_000, 2000
    codes = rng.integers(0, 65536, size=(N, 8)).astype(np.uint16)
    qtab = np.zeros((4, 8, 256), np.uint8)
    qtab[1] = 255                                    # every qd saturates at 255
    qtab[2, 0, :] = (np.arange(256) % 2) * 3         # two buckets only: 0 and 3
    qtab[3] = rng.integers(0, 2, size=(8, 256))      # ~9 buckets, huge ties
    codes[:, :] = codes[:, :]                        # keep random
    print("scan giant ties", flush=True)
    scan_vs_oracle(codes, qtab, r)
    codes[:] = 7                                     # all codes identical: one bucket holds everything
    scan_vs_oracle(codes, qtab, r)


def test_scan_selection_with_one_large_group_of_equal_candidates():
    # 2500 identical codes in the first stretch of the array share qd = 0: one (bucket, id range) group of the
    # selection exceeds what it ranks by counting, so the query is ordered by the sorting network instead;
    # a second query has the same run spread over the whole array (small groups)
    rng = np.random.default_rng(2024)
    N, r = 200_000, 3000
    codes = rng.integers(0, 65536, size=(N, 8)).astype(np.uint16)
    qtab = rng.integers(10, 58, size=(2, 8, 256)).astype(np.uint8)
    same = np.array([3, 300, 77, 1025, 9, 4242, 513, 65535], np.uint16)
    qtab[:, np.arange(8), same & 255] = 0
    codes[100:2600] = same
    print("scan with a large group of equal candidates", flush=True)
    scan_vs_oracle(codes, qtab, r)
    codes2 = codes.copy()
    codes2[100:2600] = rng.integers(0, 65536, size=(2500, 8)).astype(np.uint16)
    codes2[rng.permutation(N)[:2500]] = same
    scan_vs_oracle(codes2, qtab[1:], r)


def test_small_tables_edges_degenerate_range_and_r_beyond_n():
    rng = np.random.default_rng(5)
    m, dsub = 8, 16
    cb = torch.from_numpy((rng.normal(size=(m, 65536, dsub)) * 10).astype(np.float32)).to(DEV)
    derived = binding.derive_codebooks(cb)
    queries = torch.from_numpy((rng.normal(size=(3, m * dsub)) * 10).astype(np.float32)).to(DEV)
    dnp = oracle.derive_codebooks(to_np(cb))
    np.testing.assert_array_equal(to_np(derived), dnp)
    # (a) r beyond the number of codes: bounds use all codes
    codes_np = rng.integers(0, 65536, size=(50, m)).astype(np.uint16)
    codes = torch.from_numpy(codes_np.view(np.int16)).to(DEV).view(torch.uint16)
    qtab, bounds, small = binding.build_small_tables(queries, derived, codes, 1000, want_small=True)
    torch.cuda.synchronize()
    for q in range(3):
        D = oracle.compute_tables_f32(to_np(queries)[q], dnp)
        lo, hi = oracle.bounds(D, codes_np, 50)
        np.testing.assert_array_equal(to_np(small)[q], D)
        assert tuple(to_np(bounds)[q]) == (lo, hi)
        np.testing.assert_array_equal(to_np(qtab)[q], oracle.quantize(D, lo, hi))
    # (b) degenerate range: m = 1 and the only code seen is the arg-min entry -> qmax == qmin
    cb1 = cb[:1].contiguous(); d1 = binding.derive_codebooks(cb1)
    y1 = queries[:, :dsub].contiguous()
    D = oracle.compute_tables_f32(to_np(y1)[0], to_np(d1))
    amin = int(D.argmin())
    c1 = torch.full((10, 1), amin, dtype=torch.int16, device=DEV).view(torch.uint16)
    qtab, bounds, _ = binding.build_small_tables(y1[:1].contiguous(), d1, c1, 10)
    torch.cuda.synchronize()
    assert to_np(bounds)[0, 0] == to_np(bounds)[0, 1]
    assert (to_np(qtab) == 0).all()


def test_argument_errors_are_reported_not_launched():
    codes = torch.zeros((100, 8), dtype=torch.int16, device=DEV).view(torch.uint16)
    qtab = torch.zeros((2, 8, 256), dtype=torch.uint8, device=DEV)
    with pytest.raises(binding.DcpqError) as e:
        binding.scan_candidates(codes, qtab, 101)            # r > N
    assert e.value.code == binding.EINVAL
    with pytest.raises(binding.DcpqError) as e:
        binding.scan_candidates(codes, qtab, 10, workspace=torch.empty(256, dtype=torch.uint8, device=DEV))
    assert e.value.code == binding.EWORKSPACE
    codes3 = torch.zeros((100, 3), dtype=torch.int16, device=DEV).view(torch.uint16)
    qtab3 = torch.zeros((2, 3, 256), dtype=torch.uint8, device=DEV)
    with pytest.raises(binding.DcpqError) as e:
        binding.scan_candidates(codes3, qtab3, 10)            # m = 3 not built
    assert e.value.code == binding.EUNSUPPORTED
    codes4 = torch.zeros((100, 4), dtype=torch.int16, device=DEV).view(torch.uint16)
    qtab4 = torch.zeros((2, 4, 256), dtype=torch.uint8, device=DEV)
    with pytest.raises(binding.DcpqError) as e:
        binding.scan_candidates(codes4, qtab4, 10, mode=binding.SCAN_TILE16)   # no 16-query tile for m = 4
    assert e.value.code == binding.EUNSUPPORTED
    tables = torch.zeros((2, 8, 65536), dtype=torch.float32, device=DEV)
    cand = torch.zeros((2, 10), dtype=torch.int32, device=DEV).view(torch.uint32)
    with pytest.raises(binding.DcpqError) as e:
        binding.refine_topk(tables, codes, cand, 11)          # k > r
    assert e.value.code == binding.EINVAL


def test_determinism_and_both_algorithms_identical(case0):
    c = case0
    a_id, a_qd = binding.scan_candidates(c.codes, c.qtab, c.w.r)
    b_id, b_qd = binding.scan_candidates(c.codes, c.qtab, c.w.r)
    t_id, t_qd = binding.scan_candidates(c.codes, c.qtab, c.w.r, mode=binding.SCAN_THREE_PASS)
    torch.cuda.synchronize()
    assert torch.equal(a_id.view(torch.int32), b_id.view(torch.int32)) and torch.equal(a_qd, b_qd)
    assert torch.equal(a_id.view(torch.int32), t_id.view(torch.int32)) and torch.equal(a_qd, t_qd)


def test_scan_many_queries_ragged_tiles_and_a_few_pathological_ones():
    """Several query tiles with a ragged last tile; a handful of queries have degenerate tables whose
    candidate buffers overflow in the single pass, so they take the redo path while the rest do not."""
    rng = np.random.default_rng(321)
    N, Q, r = 300_007, 150, 1200
    codes = rng.integers(0, 65536, size=(N, 8)).astype(np.uint16)
    qtab = rng.integers(0, 48, size=(Q, 8, 256)).astype(np.uint8)
    qtab[3] = 0
    qtab[64] = 255
    qtab[149] = (rng.integers(0, 2, size=(8, 256)) * 40).astype(np.uint8)
    print("scan many queries N=%d Q=%d" % (N, Q), flush=True)
    scan_vs_oracle(codes, qtab, r)


def test_scan_random_shapes():
    """Seeded sweep of odd shapes (sizes around the group, tile, slice and queue limits) through every scan
    algorithm the shape has."""
    rng = np.random.default_rng(20260101)
    for case in range(24):
        m = int(rng.choice([4, 8, 8, 16, 32]))
        N = int(rng.choice([1, 63, 64, 65, 1023, 1025, 4097, 20_011, 65_537, 150_001]))
        Q = int(rng.choice([1, 2, 15, 16, 17, 33, 64, 65, 129]))
        r = int(min(N, rng.choice([1, 2, 63, 64, 65, 500, 3000])))
        hi = int(rng.choice([2, 8, 256 // m + 8, 256]))
        codes = rng.integers(0, 65536, size=(N, m)).astype(np.uint16)
        qtab = rng.integers(0, hi, size=(Q, m, 256)).astype(np.uint8)
        modes = [binding.SCAN_AUTO, binding.SCAN_THREE_PASS]
        if m == 8:
            modes += [binding.SCAN_TILE16, binding.SCAN_TILE32, binding.SCAN_TILE64]
        print("scan random case %d: m=%d N=%d Q=%d r=%d table values < %d" % (case, m, N, Q, r, hi), flush=True)
        scan_vs_oracle(codes, qtab, r, modes=tuple(modes))


@pytest.mark.parametrize("Q", [5, 70])
def test_scan_large_array_estimated_starting_bound(Q):
    """On a large array the single pass starts from a bound estimated from a sample (the sample's count
    scaled to the array), not from the sample's own r-th smallest; ids stay global, every code is scanned
    exactly once (all tiles, ragged last workgroup)."""
    rng = np.random.default_rng(77 + Q)
    N, r = 4_200_003, 700
    codes = rng.integers(0, 65536, size=(N, 8)).astype(np.uint16)
    qtab = rng.integers(0, 40, size=(Q, 8, 256)).astype(np.uint8)
    print("scan large-array case N=%d Q=%d r=%d" % (N, Q, r), flush=True)
    scan_vs_oracle(codes, qtab, r, modes=(binding.SCAN_AUTO, binding.SCAN_TILE16, binding.SCAN_TILE64))


def test_scan_pilot_pass_starting_bound():
    """A batch large enough for the sample to be read in two stages: the histogram pass over one run in 16, then
    the single-pass kernel itself counting the whole sample below the bound that gives (runs addressed by
    stride, a last run cut by the end of the array is possible, nothing stored), then the scan proper."""
    rng = np.random.default_rng(4242)
    N, Q, r = 1_200_003, 1000, 700
    for mode in (binding.SCAN_AUTO, binding.SCAN_TILE16, binding.SCAN_TILE32):
        assert binding.scan_plan(N, 8, Q, r, mode)["pilot_every"] == 16
    codes = rng.integers(0, 65536, size=(N, 8)).astype(np.uint16)
    qtab = rng.integers(0, 40, size=(Q, 8, 256)).astype(np.uint8)
    qtab[5] = 0                       # every code ties at 0
    qtab[6] = 255                     # every code saturates
    print("scan pilot-pass case N=%d Q=%d r=%d" % (N, Q, r), flush=True)
    scan_vs_oracle(codes, qtab, r, modes=(binding.SCAN_AUTO, binding.SCAN_TILE16, binding.SCAN_TILE32))


@pytest.mark.parametrize("m,Q", [(4, 2000), (16, 500), (32, 250)])
def test_scan_pilot_pass_other_code_widths(m, Q):
    """The pilot pass with the dense matrix instruction (m = 4) and with the 32- and 16-query tiles of m = 16, 32."""
    rng = np.random.default_rng(4300 + m)
    N, r = 300_007, 700
    assert binding.scan_plan(N, m, Q, r)["pilot_every"] == 16
    codes = rng.integers(0, 65536, size=(N, m)).astype(np.uint16)
    qtab = rng.integers(0, 320 // m, size=(Q, m, 256)).astype(np.uint8)
    print("scan pilot-pass case m=%d N=%d Q=%d r=%d" % (m, N, Q, r), flush=True)
    scan_vs_oracle(codes, qtab, r, modes=(binding.SCAN_AUTO,))


@pytest.mark.parametrize("N,Q,pilot", [(4_200_003, 130, False), (300_003, 1000, True)])
def test_scan_estimated_bound_too_low_is_redone(N, Q, pilot):
    """The estimated starting bound fails when the sample misrepresents the array: here the near codes sit
    exactly in the runs of 256 codes, evenly spread, that the sample reads, so the estimate puts r codes
    below a bucket that holds fewer in the whole array.  Such queries (the even ones here; the odd ones'
    tables spread the near codes over half as many buckets, so their first bucket does hold r) must come
    out exact all the same: the selection sees fewer than r candidates and has them redone.  Both ways of
    reading the sample are covered."""
    rng = np.random.default_rng(5150)
    r = 700
    plan = binding.scan_plan(N, 8, Q, r)
    runs, stride = plan["sample_runs"], plan["sample_stride"]
    # a sample well inside the array; with the larger batch it is read in two stages (histogram of one run in 16,
    # then the pilot pass of the single-pass kernel), with the smaller one by the histogram pass alone
    assert runs * 256 * 4 <= N and plan["pilot_every"] == (16 if pilot else 1)
    # the near codes (all in the sample) spread over 100 buckets for the even queries: fewer than r in the first
    # bucket, which is nevertheless where the estimate starts (it expects r * sample / N + slack codes there)
    assert runs * 256 / 100 < r < runs * 256 / 50
    pos = (np.arange(runs, dtype=np.int64)[:, None] * stride + np.arange(256)[None, :]).ravel()
    codes = rng.integers(0, 65536, size=(N, 8)).astype(np.uint16)
    low0 = rng.integers(200, 256, size=N)
    low0[pos] = rng.integers(0, 100, size=pos.size)
    codes[:, 0] = (codes[:, 0] & 0xFF00) | low0.astype(np.uint16)
    qtab = np.zeros((Q, 8, 256), dtype=np.uint8)
    qtab[0::2, 0, :] = np.arange(256, dtype=np.uint8)[None, :]            # qd = the low byte: ~655 codes per bucket
    qtab[1::2, 0, :] = (np.arange(256) // 2).astype(np.uint8)[None, :]    # ~1310 per bucket
    binding.profile_enable(True)
    try:
        scan_vs_oracle(codes, qtab, r, modes=(binding.SCAN_AUTO,))
        stages = binding.profile_read()
    finally:
        binding.profile_enable(False)
    print("redo stages (ms, launches): hist+sample %s, tie count %s, collect %s"
          % (stages.get("scan_hist"), stages.get("scan_tiecount"), stages.get("scan_collect")), flush=True)
