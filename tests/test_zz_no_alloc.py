"""The scan entry point that allocates nothing (static scratch array inside the library) against
the entry point with a caller-provided workspace: same candidates, bit for bit, on two calls in a
row, the second with a smaller problem (the array keeps the first call's contents)."""
import pytest
import torch

from paper_1905_06900_amd import binding, synth

pytestmark = pytest.mark.gpu


def _case(N, Q, r, seed_offset):
    dev = "cuda:0"
    w = synth.scaled(synth.WORKLOADS[1], N=N, Q=Q, r=r)
    w = synth.Workload(**{**w.__dict__, "seed": w.seed + seed_offset, "data": "deep_random_codes", "dsub": 12})
    d = synth.make_flat(w, dev)
    derived = binding.derive_codebooks(d["codebooks"])
    qtab, _, _ = binding.build_small_tables(d["queries"], derived, d["codes"], r)
    return d["codes"], qtab


def _both(codes, qtab, r):
    nq = qtab.shape[0]
    want_id, want_qd = binding.scan_candidates(codes, qtab, r)
    got_id = torch.full((nq, r), 0xDEADBEEF, dtype=torch.uint32, device=codes.device)
    got_qd = torch.full((nq, r), 0xEE, dtype=torch.uint8, device=codes.device)
    binding.scan_candidates_static(codes, qtab, r, got_id, got_qd)
    torch.cuda.synchronize()
    assert torch.equal(got_id.view(torch.int32), want_id.view(torch.int32))
    assert torch.equal(got_qd, want_qd)


def test_static_scratch_scan_matches_the_workspace_scan_twice():
    assert binding.lib().dcpq_static_scratch_bytes() == 64 << 20
    codes, qtab = _case(300_017, 70, 1500, 0)        # two query tiles of 64, ragged tail of codes
    assert binding.scan_workspace_bytes(codes.shape[0], codes.shape[1], qtab.shape[0], 1500) <= 64 << 20
    _both(codes, qtab, 1500)
    codes2, qtab2 = _case(40_003, 5, 100, 1)         # smaller: the array still holds the first call's data
    _both(codes2, qtab2, 100)


def test_static_scratch_scan_refuses_what_does_not_fit():
    codes, qtab = _case(100_000, 8, 100, 2)
    big_q = qtab.repeat(64, 1, 1).contiguous()       # 512 queries x r = 50000 does not fit 64 MiB
    r = 50_000
    assert binding.scan_workspace_bytes(codes.shape[0], codes.shape[1], big_q.shape[0], r) > 64 << 20
    ids = torch.empty((big_q.shape[0], r), dtype=torch.uint32, device=codes.device)
    qd = torch.empty((big_q.shape[0], r), dtype=torch.uint8, device=codes.device)
    with pytest.raises(binding.DcpqError) as e:
        binding.scan_candidates_static(codes, big_q, r, ids, qd)
    assert e.value.code == binding.EWORKSPACE
