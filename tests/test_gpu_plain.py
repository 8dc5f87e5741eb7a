"""GPU parity tests of the conventional single-pass search (Alg. 1): every code scored with the
full floating-point tables, once as a 16-bit product quantizer and once as an 8-bit one, against
the oracle's exhaustive search."""
import numpy as np
import pytest
import torch

import oracle
from paper_1905_06900_amd import binding, synth
from parity import to_np, assert_topk_matches

pytestmark = pytest.mark.gpu

DEV = "cuda"


def check_against_exhaustive(tables, cb, codes, queries, k, b, qsel):
    ids, dist = binding.plain_search(tables, codes, k)
    torch.cuda.synchronize()
    ids, dist = to_np(ids), to_np(dist)
    cb_np, q_np = to_np(cb), to_np(queries)
    codes_np = to_np(codes).astype(np.uint16)
    ref_ids, ref_dist = oracle.search_exhaustive(cb_np, codes_np, q_np[qsel], k, b=b)
    for a, q in enumerate(qsel):
        exact = oracle.refine(q_np[q], cb_np, codes_np, ids[q], b=b)
        assert_topk_matches(ids[q], dist[q], ref_ids[a], ref_dist[a], exact, tag="query %d" % q)


@pytest.mark.parametrize("k", [1, 100, 768])
def test_plain_16_bit_m4_against_exhaustive_oracle(k):
    w = synth.scaled(synth.WORKLOADS[0], N=150_003, Q=21, r=1000)
    print("plain 16-bit: cfg0 recipe N=%d Q=%d k=%d" % (w.N, w.Q, k), flush=True)
    d = synth.make_flat(w, DEV)
    tables = binding.build_tables(d["queries"], d["codebooks"])
    check_against_exhaustive(tables, d["codebooks"], d["codes"], d["queries"], k, 16, [0, 7, 8, 20])


@pytest.mark.parametrize("m,dsub,N,Q", [(8, 12, 90_001, 19), (16, 8, 20_011, 9)])
def test_plain_8_bit_against_exhaustive_oracle(m, dsub, N, Q):
    print("plain 8-bit: m=%d dsub=%d N=%d Q=%d" % (m, dsub, N, Q), flush=True)
    g = torch.Generator(device=DEV); g.manual_seed(4100 + m)
    cb = 0.3 * torch.randn((m, 256, dsub), generator=g, device=DEV, dtype=torch.float32)
    codes = torch.randint(0, 256, (N, m), generator=g, device=DEV, dtype=torch.uint8)
    queries = 0.3 * torch.randn((Q, m * dsub), generator=g, device=DEV, dtype=torch.float32)
    tables = binding.build_tables_n(queries, cb)
    T = to_np(tables)
    want = oracle.compute_tables_f64(to_np(queries)[3], to_np(cb))
    np.testing.assert_allclose(T[3], want, rtol=1e-6, atol=1e-30)
    check_against_exhaustive(tables, cb, codes, queries, 100, 8, [0, 8, Q - 1])


def test_plain_search_with_fewer_codes_than_a_batch_and_k_equal_n():
    g = torch.Generator(device=DEV); g.manual_seed(77)
    m, dsub, N, Q = 4, 6, 100, 3
    cb = torch.randn((m, 256, dsub), generator=g, device=DEV, dtype=torch.float32)
    codes = torch.randint(0, 256, (N, m), generator=g, device=DEV, dtype=torch.uint8)
    queries = torch.randn((Q, m * dsub), generator=g, device=DEV, dtype=torch.float32)
    tables = binding.build_tables_n(queries, cb)
    ids, dist = binding.plain_search(tables, codes, N)
    torch.cuda.synchronize()
    ids = to_np(ids)
    for q in range(Q):
        assert sorted(ids[q].tolist()) == list(range(N))
    check_against_exhaustive(tables, cb, codes, queries, N, 8, [0, 1, 2])


def test_plain_search_rejects_k_above_its_limit():
    tables = torch.zeros((1, 4, 256), dtype=torch.float32, device=DEV)
    codes = torch.zeros((2000, 4), dtype=torch.uint8, device=DEV)
    with pytest.raises(binding.DcpqError):
        binding.plain_search(tables, codes, 769, workspace=torch.empty(1 << 20, dtype=torch.uint8, device=DEV))
