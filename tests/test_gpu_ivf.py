"""GPU parity tests of the inverted-index variant, stage by stage, through the C ABI.

The oracle takes the probed lists as an input, so the Index step is compared on its own (sets of
lists and their order, with near-ties of the coarse distance allowed) and the library's own probe
lists are then handed to the oracle: everything after them must match bit for bit (bounds, 8-bit
tables, candidate ids / integer distances / counts) or within 1e-5 (re-ranked distances)."""
import numpy as np
import pytest
import torch

import oracle
from paper_1905_06900_amd import binding, synth
from parity import to_np, assert_topk_matches, REL_TOL

pytestmark = pytest.mark.gpu
DEV = "cuda"


def run_ivf_case(d, nprobe, r, k, check_probe=True, plane=False, fused=False):
    """plane: the scan reads the low-byte plane instead of the codes; fused: the final ids and distances come
    from the one-call search (whose probe lists are the staged ones: same kernels, same inputs)."""
    cb, coarse, offsets, codes, queries = d["codebooks"], d["coarse"], d["offsets"], d["codes"], d["queries"]
    derived = binding.derive_codebooks(cb)
    low = binding.pack_low_bytes(codes) if plane else None
    probe = binding.ivf_probe(queries, coarse, nprobe)
    qtab, bounds = binding.ivf_build_small_tables(queries, coarse, probe, derived, codes, offsets, r)
    # the variant that keeps the entries between its passes gives the same bytes
    qtab2, bounds2 = binding.ivf_build_small_tables(queries, coarse, probe, derived, codes, offsets, r, keep_entries=True)
    assert torch.equal(qtab, qtab2) and torch.equal(bounds, bounds2)
    cand_id, cand_qd, count = binding.ivf_scan_candidates(low if plane else codes, offsets, probe, qtab, r)
    ids, dist = binding.ivf_refine_topk(queries, coarse, cb, codes, offsets, probe, cand_id, k)
    if fused:
        ids, dist = binding.ivf_search(queries, coarse, cb, derived, codes, offsets, nprobe, r, k, plane=low)
    torch.cuda.synchronize()

    cb_np, coarse_np, off_np = to_np(cb), to_np(coarse), to_np(offsets)
    codes_np, q_np, probe_np = to_np(codes), to_np(queries), to_np(probe)
    nq = q_np.shape[0]
    if check_probe:
        want = oracle.ivf_probe(q_np, coarse_np, nprobe)
        dd = ((q_np[:, None, :].astype(np.float64) - coarse_np[None, :, :].astype(np.float64)) ** 2).sum(-1) \
            if coarse_np.shape[0] * nq < 4_000_000 else None
        for q in range(nq):
            assert len(set(probe_np[q].tolist())) == nprobe
            if (probe_np[q] != want[q]).any():
                assert dd is not None
                # only near-ties of the coarse distance may reorder or swap lists
                np.testing.assert_allclose(dd[q, probe_np[q]], dd[q, want[q]], rtol=1e-6)
    der_ref = oracle.derive_codebooks(cb_np)
    np.testing.assert_array_equal(to_np(derived), der_ref)
    ref = oracle.search_ivf(cb_np, der_ref, codes_np, off_np, coarse_np, q_np, probe_np, r, k)
    np.testing.assert_array_equal(to_np(bounds), ref["bounds"], err_msg="bounds")
    np.testing.assert_array_equal(to_np(qtab), ref["qtab"], err_msg="quantized tables")
    np.testing.assert_array_equal(to_np(count), ref["count"], err_msg="count")
    np.testing.assert_array_equal(to_np(cand_id), ref["cand_id"], err_msg="candidate ids")
    np.testing.assert_array_equal(to_np(cand_qd), ref["cand_qd"], err_msg="candidate qd")
    ids_np, dist_np = to_np(ids), to_np(dist)
    for q in range(nq):
        kk = min(k, int(ref["count"][q]))
        assert (ids_np[q, kk:] == binding.PAD_ID).all() and np.isinf(dist_np[q, kk:]).all()
        if kk == 0:
            continue
        # exact distance of the ids the library returned: Eq. 3 on the residual of their list
        list_of = np.searchsorted(off_np, ids_np[q, :kk].astype(np.int64), side="right") - 1
        cen = np.stack([np.concatenate([cb_np[j][codes_np[i, j]] for j in range(cb_np.shape[0])]) for i in ids_np[q, :kk]])
        exact = ((q_np[q].astype(np.float64)[None, :] - coarse_np[list_of].astype(np.float64) - cen.astype(np.float64)) ** 2).sum(1)
        assert_topk_matches(ids_np[q, :kk], dist_np[q, :kk], ref["ids"][q, :kk], ref["dist"][q, :kk], exact,
                            cand_ref=ref["cand_id"][q][:int(ref["count"][q])], tag="query %d" % q)
    return ref


def test_ivf_scaled_cfg3_recipe():
    w = synth.scaled(synth.WORKLOADS[3], N=300_007, Q=23, r=500, nlist=512, nprobe=16)
    print("ivf case: cfg3 recipe nlist=512 N=300007 Q=23 nprobe=16 r=500", flush=True)
    d = synth.make_ivf(w, DEV)
    run_ivf_case(d, w.nprobe, w.r, w.k)


def test_ivf_nprobe_64_many_lists_and_large_r():
    w = synth.scaled(synth.WORKLOADS[3], N=500_000, Q=9, r=9000, nlist=4096, nprobe=64)
    print("ivf case: nlist=4096 N=500000 Q=9 nprobe=64 r=9000 (sort spills)", flush=True)
    d = synth.make_ivf(w, DEV)
    run_ivf_case(d, w.nprobe, w.r, 100)


def test_ivf_short_and_empty_lists_pad_the_outputs():
    w = synth.scaled(synth.WORKLOADS[3], N=3000, Q=7, r=300, nlist=64, nprobe=5)
    d = synth.make_ivf(w, DEV)
    # most lists tiny or empty, a few large
    sizes = torch.zeros(64, dtype=torch.int64)
    sizes[::7] = 3; sizes[5] = 2000; sizes[40] = 3000 - 2000 - int(sizes.sum()) + 2000 - 2000
    sizes[40] = 3000 - int(sizes.sum()) + int(sizes[40])
    off = torch.zeros(65, dtype=torch.int64); off[1:] = torch.cumsum(sizes, 0)
    assert int(off[-1]) == 3000
    d["offsets"] = off.to(DEV)
    print("ivf case: short and empty lists", flush=True)
    ref = run_ivf_case(d, 5, 300, 40)
    assert (ref["count"] < 300).any()


def test_ivf_all_lists_probed_identical_centres_ties_by_id():
    w = synth.scaled(synth.WORKLOADS[3], N=20_000, Q=5, r=700, nlist=16, nprobe=16)
    d = synth.make_ivf(w, DEV)
    d["coarse"] = torch.ones_like(d["coarse"])          # every coarse distance ties: probe order = list id
    print("ivf case: identical centres, nprobe = nlist", flush=True)
    run_ivf_case(d, 16, 700, 60)
    probe = to_np(binding.ivf_probe(d["queries"], d["coarse"], 16))
    assert (probe == np.arange(16)[None, :]).all()


@pytest.mark.parametrize("m,dsub", [(1, 128), (2, 64), (4, 32), (16, 8), (32, 4)])
def test_ivf_other_code_shapes(m, dsub):
    """The inverted-index path for every supported m besides the recipe's 8 (the recipe's 128-dimensional vectors split other ways)."""
    from dataclasses import replace
    w = replace(synth.scaled(synth.WORKLOADS[3], N=60_013, Q=11, r=300, nlist=128, nprobe=9), m=m, dsub=dsub)
    print("ivf case: m=%d dsub=%d N=%d Q=%d nlist=%d nprobe=%d r=%d" % (m, dsub, w.N, w.Q, w.nlist, w.nprobe, w.r),
          flush=True)
    d = synth.make_ivf(w, DEV)
    run_ivf_case(d, w.nprobe, w.r, 50)


def test_ivf_argument_errors():
    q = torch.zeros((2, 128), device=DEV); coarse = torch.zeros((8, 128), device=DEV)
    with pytest.raises(binding.DcpqError) as e:
        binding.ivf_probe(q, coarse, 9)                  # nprobe > nlist
    assert e.value.code == binding.EINVAL
    coarse = torch.zeros((1024, 128), device=DEV)
    with pytest.raises(binding.DcpqError) as e:
        binding.ivf_probe(q, coarse, 600)                # above the supported nprobe
    assert e.value.code == binding.EUNSUPPORTED


def test_low_byte_plane_scan_against_the_oracle():
    """pack_low_bytes is the low byte of every sub-code, and the scan of probed lists reading the plane gives the
    oracle's candidate ids / integer distances / counts (ragged N, padded lists)."""
    for (N, Q, r, nlist, nprobe) in [(300_007, 23, 500, 512, 16), (3001, 7, 300, 64, 5)]:
        w = synth.scaled(synth.WORKLOADS[3], N=N, Q=Q, r=r, nlist=nlist, nprobe=nprobe)
        print("ivf plane case: N=%d Q=%d r=%d nlist=%d nprobe=%d" % (N, Q, r, nlist, nprobe), flush=True)
        d = synth.make_ivf(w, DEV)
        plane = binding.pack_low_bytes(d["codes"])
        torch.cuda.synchronize()
        np.testing.assert_array_equal(to_np(plane), (to_np(d["codes"]) & 255).astype(np.uint8))
        run_ivf_case(d, nprobe, r, 50, plane=True)


def test_ivf_search_in_one_call_against_the_oracle():
    for use_plane in (False, True):
        w = synth.scaled(synth.WORKLOADS[3], N=200_003, Q=19, r=400, nlist=256, nprobe=12)
        print("ivf fused search: N=%d Q=%d plane=%s" % (w.N, w.Q, use_plane), flush=True)
        d = synth.make_ivf(w, DEV)
        run_ivf_case(d, w.nprobe, w.r, w.k, plane=use_plane, fused=True)
    # a workspace one byte short is refused, nothing is launched
    cb, q = d["codebooks"], d["queries"]
    need = binding.ivf_search_workspace_bytes(q.shape[0], 256, 12, 8, 400)
    with pytest.raises(binding.DcpqError) as e:
        binding.ivf_search(q, d["coarse"], cb, binding.derive_codebooks(cb), d["codes"], d["offsets"], 12, 400, 100,
                           workspace=torch.empty(need - 256, dtype=torch.uint8, device=DEV))
    assert e.value.code == binding.EWORKSPACE


@pytest.mark.parametrize("m", [1, 2, 4, 16, 32])
def test_low_byte_plane_every_m(m):
    rng = np.random.default_rng(m)
    n = 10_003
    codes = torch.from_numpy(rng.integers(0, 65536, size=(n, m)).astype(np.uint16).view(np.int16)).to(DEV).view(torch.uint16)
    plane = binding.pack_low_bytes(codes)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_np(plane), (to_np(codes) & 255).astype(np.uint8))
