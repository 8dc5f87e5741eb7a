"""GPU parity at the full sizes of the five benchmark workloads.

The whole batch runs through the fused entry point in the launch configuration bench.py times;
the CPU oracle, which needs about a second per query at these sizes, checks a sample of the
queries one by one: candidate sets and integer tables bit for bit (staged calls on the sampled
queries), and the final top-k of the full batch at the sampled positions."""
import numpy as np
import pytest
import torch

import oracle
from paper_1905_06900_amd import binding, synth
from parity import to_np, assert_topk_matches
from test_gpu_ivf import run_ivf_case

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]
DEV = "cuda"


def full_flat(cfg, nsample):
    w = synth.WORKLOADS[cfg]
    print("full-size case: %s N=%d Q=%d r=%d k=%d, oracle on %d sampled queries" % (w.name, w.N, w.Q, w.r, w.k, nsample), flush=True)
    d = synth.make_flat(w, DEV)
    cb, codes, queries = d["codebooks"], d["codes"], d["queries"]
    derived = binding.derive_codebooks(cb)
    ids, dist = binding.search(queries, cb, derived, codes, w.r, w.k)          # the whole batch, as timed
    torch.cuda.synchronize()
    print("  fused search done", flush=True)
    rng = np.random.default_rng(cfg)
    sel = np.sort(rng.choice(w.Q, size=min(nsample, w.Q), replace=False))
    qs = queries[torch.from_numpy(sel).to(DEV)].contiguous()
    qtab, bounds, small = binding.build_small_tables(qs, derived, codes, w.r, want_small=True)
    cand_id, cand_qd = binding.scan_candidates(codes, qtab, w.r)
    torch.cuda.synchronize()
    cb_np, codes_np, q_np = to_np(cb), to_np(codes), to_np(qs)
    der_ref = oracle.derive_codebooks(cb_np)
    np.testing.assert_array_equal(to_np(derived), der_ref)
    ref = oracle.search_flat(cb_np, der_ref, codes_np, q_np, w.r, w.k)
    print("  oracle done", flush=True)
    np.testing.assert_array_equal(to_np(small), ref["small"], err_msg="small tables")
    np.testing.assert_array_equal(to_np(bounds), ref["bounds"], err_msg="bounds")
    np.testing.assert_array_equal(to_np(qtab), ref["qtab"], err_msg="quantized tables")
    np.testing.assert_array_equal(to_np(cand_id), ref["cand_id"], err_msg="candidate ids")
    np.testing.assert_array_equal(to_np(cand_qd), ref["cand_qd"], err_msg="candidate qd")
    ids_np, dist_np = to_np(ids)[sel], to_np(dist)[sel]
    for a in range(len(sel)):
        exact = oracle.refine(q_np[a], cb_np, codes_np, ids_np[a])
        assert_topk_matches(ids_np[a], dist_np[a], ref["ids"][a], ref["dist"][a], exact, cand_ref=ref["cand_id"][a],
                            tag="%s query %d" % (w.name, sel[a]))


def test_cfg0_full_all_queries():
    full_flat(0, 100)


def test_cfg1_full_sift_encoded():
    full_flat(1, 24)


def test_cfg2_full_headline_workload():
    full_flat(2, 16)


def test_cfg4_full_gist_16x16():
    full_flat(4, 16)


def test_cfg3_full_ivf_one_billion_codes():
    w = synth.WORKLOADS[3]
    nsample = 48
    print("full-size case: %s N=%d nlist=%d nprobe=%d r=%d, %d of %d queries" % (w.name, w.N, w.nlist, w.nprobe, w.r, nsample, w.Q), flush=True)
    d = synth.make_ivf(w, DEV)
    # the timed configuration: the whole batch through every stage
    cb, coarse, offsets, codes, queries = d["codebooks"], d["coarse"], d["offsets"], d["codes"], d["queries"]
    derived = binding.derive_codebooks(cb)
    probe = binding.ivf_probe(queries, coarse, w.nprobe)
    qtab, bounds = binding.ivf_build_small_tables(queries, coarse, probe, derived, codes, offsets, w.r)
    cand_id, cand_qd, count = binding.ivf_scan_candidates(codes, offsets, probe, qtab, w.r)
    ids, dist = binding.ivf_refine_topk(queries, coarse, cb, codes, offsets, probe, cand_id, w.k)
    torch.cuda.synchronize()
    print("  full batch done", flush=True)
    assert int(count.view(torch.int32).min()) == w.r
    full_ids = to_np(ids)
    del qtab, cand_id, cand_qd, ids, dist
    # the sampled queries again on their own, against the oracle (host copy of the 16 GB of codes)
    sel = np.sort(np.random.default_rng(3).choice(w.Q, size=nsample, replace=False))
    d["queries"] = queries[torch.from_numpy(sel).to(DEV)].contiguous()
    run_ivf_case(d, w.nprobe, w.r, w.k, check_probe=False)
    # probe lists of the sampled queries against exact fp64 coarse distances (near-ties allowed)
    q_np, coarse_np = to_np(d["queries"]), to_np(coarse)
    want = oracle.ivf_probe(q_np, coarse_np, w.nprobe)
    got = to_np(probe)[sel]
    for a in range(nsample):
        if (got[a] != want[a]).any():
            da = ((coarse_np[got[a]].astype(np.float64) - q_np[a]) ** 2).sum(1)
            dw = ((coarse_np[want[a]].astype(np.float64) - q_np[a]) ** 2).sum(1)
            np.testing.assert_allclose(da, dw, rtol=1e-6)
    # the batch run and the sampled run agree
    ids_s, _ = binding.ivf_refine_topk(d["queries"], coarse, cb, codes, offsets,
                                       binding.ivf_probe(d["queries"], coarse, w.nprobe),
                                       binding.ivf_scan_candidates(codes, offsets, binding.ivf_probe(d["queries"], coarse, w.nprobe),
                                                                   binding.ivf_build_small_tables(d["queries"], coarse, binding.ivf_probe(d["queries"], coarse, w.nprobe), derived, codes, offsets, w.r)[0], w.r)[0],
                                       w.k)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_np(ids_s), full_ids[sel])
