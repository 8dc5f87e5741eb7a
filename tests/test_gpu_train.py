"""GPU parity tests of training and encoding (Sec. 3.2, Alg. 2) against the oracle: nearest-centroid
assignment and encoding, k-means, same-size k-means (balanced assignment in rounds), the final
codebook order, and all of Alg. 2 in one call."""
import numpy as np
import pytest
import torch

import oracle
from paper_1905_06900_amd import binding, synth
from parity import to_np

pytestmark = pytest.mark.gpu

DEV = "cuda"


def gen(seed):
    g = torch.Generator(device=DEV); g.manual_seed(seed)
    return g


def check_labels(labels, points, cb, ref_labels, tag):
    """Labels equal the oracle's wherever the oracle's best and second-best centroids are apart; where they
    are closer than 1e-9 relative (the two sides add their double-precision terms in different orders) the
    chosen centroid must be as near as the best."""
    labels = labels.astype(np.int64); ref_labels = ref_labels.astype(np.int64)
    diff = np.nonzero(labels != ref_labels)[0]
    assert len(diff) <= max(1, len(labels) // 1000), tag + ": %d labels differ" % len(diff)
    for i in diff:
        x = points[i].astype(np.float64)
        da = ((x - cb[labels[i]].astype(np.float64)) ** 2).sum()
        db = ((x - cb[ref_labels[i]].astype(np.float64)) ** 2).sum()
        assert abs(da - db) <= 1e-9 * max(db, 1e-300), tag + ": point %d got a farther centroid" % i


@pytest.mark.parametrize("n,m,dsub,ncent", [(1000, 2, 6, 1000), (333, 1, 13, 77), (4097, 4, 4, 256), (50, 1, 128, 300)])
def test_assign_against_the_oracle(n, m, dsub, ncent):
    print("assign n=%d m=%d dsub=%d ncent=%d" % (n, m, dsub, ncent), flush=True)
    g = gen(100 + n)
    pts = torch.randn((n, m * dsub), generator=g, device=DEV)
    cb = torch.randn((m, ncent, dsub), generator=g, device=DEV)
    cb[:, 5] = cb[:, 3]                                          # a duplicate centroid: the smaller index must win
    pts[7, :dsub] = cb[0, 5]
    labels, dist = binding.assign(pts, cb, want_dist=True)
    torch.cuda.synchronize()
    labels, dist, p_np, c_np = to_np(labels), to_np(dist), to_np(pts), to_np(cb)
    assert labels[7, 0] == 3
    for j in range(m):
        ref, rd = oracle.assign(p_np[:, j * dsub:(j + 1) * dsub], c_np[j], want_dist=True)
        check_labels(labels[:, j], p_np[:, j * dsub:(j + 1) * dsub], c_np[j], ref, "sub-quantizer %d" % j)
        # (a point that IS a centroid: the expanded form ||x||^2 + ||c||^2 - 2<x, c> leaves a rounding residue of
        # the order of 1e-16 times the norms instead of an exact zero)
        np.testing.assert_allclose(dist[:, j], rd, rtol=1e-5, atol=1e-12 * float((p_np.astype(np.float64) ** 2).sum(1).max()))


@pytest.mark.parametrize("b", [16, 8])
def test_encode_against_the_oracle(b):
    m, dsub, n = (4, 8, 3000) if b == 16 else (8, 4, 20000)
    print("encode b=%d m=%d dsub=%d n=%d" % (b, m, dsub, n), flush=True)
    cb = synth.hierarchical_codebooks(m, dsub, b, 4, lambda shape, gg: 3.0 * torch.randn(
        shape, generator=gg, device=DEV, dtype=torch.float32), 0.5, DEV, 4242 + b)
    g = gen(77 + b)
    codes_true = torch.randint(0, 1 << b, (n, m), generator=g, device=DEV)
    x = torch.cat([cb[j][codes_true[:, j]] for j in range(m)], dim=1) + 0.2 * torch.randn((n, m * dsub), generator=g, device=DEV)
    codes = binding.encode(x, cb)
    torch.cuda.synchronize()
    assert codes.dtype == (torch.uint16 if b == 16 else torch.uint8)
    codes, x_np, cb_np = to_np(codes), to_np(x), to_np(cb)
    ref = oracle.encode(x_np, cb_np)
    for j in range(m):
        check_labels(codes[:, j], x_np[:, j * dsub:(j + 1) * dsub], cb_np[j], ref[:, j], "sub-quantizer %d" % j)
    # decodable vectors come back as their own codes
    exact = torch.cat([cb[j][codes_true[:50, j]] for j in range(m)], dim=1).contiguous()
    back = to_np(binding.encode(exact, cb)).astype(np.int64)
    xe = to_np(exact)
    for j in range(m):
        check_labels(back[:, j], xe[:, j * dsub:(j + 1) * dsub], cb_np[j], to_np(codes_true[:50, j]), "decodable, %d" % j)


def test_kmeans_against_the_oracle():
    n, d, k = 20000, 8, 256
    print("kmeans n=%d d=%d k=%d" % (n, d, k), flush=True)
    g = gen(5)
    means = 4.0 * torch.randn((64, d), generator=g, device=DEV)
    x = means[torch.randint(0, 64, (n,), generator=g, device=DEV)] + torch.randn((n, d), generator=g, device=DEV)
    init = x[:k].clone()
    for iters in (0, 1, 4):
        cent, labels = binding.kmeans(x, init, iters)
        torch.cuda.synchronize()
        rc, rl = oracle.kmeans(to_np(x), to_np(init), iters)
        np.testing.assert_allclose(to_np(cent), rc, rtol=1e-5, atol=1e-6, err_msg="centroids after %d iterations" % iters)
        check_labels(to_np(labels), to_np(x), rc, rl, "labels after %d iterations" % iters)


def test_kmeans_centroid_without_members_keeps_its_value():
    x = torch.tensor([[0.0, 0.0], [1.0, 0.0], [2.0, 0.0], [3.0, 0.0]], device=DEV)
    init = torch.tensor([[1.0, 0.0], [100.0, 0.0]], device=DEV)
    cent, labels = binding.kmeans(x, init, 3)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_np(labels), [0, 0, 0, 0])
    np.testing.assert_array_equal(to_np(cent), np.array([[1.5, 0.0], [100.0, 0.0]], np.float32))


@pytest.mark.parametrize("n,d,kbar,iters", [(4096, 6, 16, 2), (1024, 3, 256, 1), (65536, 12, 256, 1)])
def test_same_size_kmeans_against_the_oracle(n, d, kbar, iters):
    print("same-size k-means n=%d d=%d kbar=%d iters=%d" % (n, d, kbar, iters), flush=True)
    g = gen(900 + kbar + n)
    means = 3.0 * torch.randn((40, d), generator=g, device=DEV)
    # lopsided on purpose: most points around a few of the means, so that many groups overflow
    pick = (torch.rand((n,), generator=g, device=DEV) ** 3 * 40).long().clamp(max=39)
    p = (means[pick] + 0.7 * torch.randn((n, d), generator=g, device=DEV)).contiguous()
    init = p[:kbar].clone()
    cent, labels = binding.kmeans_same_size(p, init, iters)
    torch.cuda.synchronize()
    labels, cent = to_np(labels), to_np(cent)
    np.testing.assert_array_equal(np.bincount(labels, minlength=kbar), np.full(kbar, n // kbar))
    rc, rl = oracle.kmeans_same_size(to_np(p), to_np(init), iters)
    np.testing.assert_array_equal(labels, rl.astype(np.int32))
    np.testing.assert_allclose(cent, rc, rtol=1e-5, atol=1e-6)


def test_final_codebook_against_the_oracle():
    g = gen(31)
    for b, bbar, d in [(8, 3, 5), (16, 8, 12), (8, 8, 4)]:
        k, kbar = 1 << b, 1 << bbar
        labels = torch.arange(kbar, device=DEV, dtype=torch.int32).repeat_interleave(k // kbar)[torch.randperm(k, generator=g, device=DEV)].contiguous()
        temp = torch.randn((k, d), generator=g, device=DEV)
        final, perm = binding.build_final_codebook(temp, labels, bbar)
        torch.cuda.synchronize()
        rf, rp = oracle.build_final_codebook(to_np(temp), to_np(labels), bbar)
        np.testing.assert_array_equal(to_np(perm), rp.astype(np.int32))
        np.testing.assert_array_equal(to_np(final), rf)


def test_all_of_alg2_in_one_call_against_the_oracle_steps():
    m, dsub, b, bbar, n, iters, ss = 2, 4, 8, 4, 6000, 3, 2
    print("build_quantizers m=%d dsub=%d b=%d bbar=%d n=%d" % (m, dsub, b, bbar, n), flush=True)
    g = gen(64)
    means = 5.0 * torch.randn((300, m * dsub), generator=g, device=DEV)
    x = (means[torch.randint(0, 300, (n,), generator=g, device=DEV)] + torch.randn((n, m * dsub), generator=g, device=DEV)).contiguous()
    init = torch.stack([x[:1 << b, j * dsub:(j + 1) * dsub] for j in range(m)]).contiguous()
    cb, derived = binding.build_quantizers(x, init, bbar, iters, ss)
    torch.cuda.synchronize()
    x_np, init_np = to_np(x), to_np(init)
    for j in range(m):
        temp, _ = oracle.kmeans(np.ascontiguousarray(x_np[:, j * dsub:(j + 1) * dsub]), init_np[j], iters)
        cbar, lab = oracle.kmeans_same_size(temp, temp[:1 << bbar].copy(), ss)
        final, _ = oracle.build_final_codebook(temp, lab, bbar)
        np.testing.assert_allclose(to_np(cb)[j], final, rtol=1e-5, atol=1e-6, err_msg="final codebook %d" % j)
        np.testing.assert_allclose(to_np(derived)[j], cbar, rtol=1e-5, atol=1e-6, err_msg="derived codebook %d" % j)
    # the derived codebooks are those of the search path, and the search runs on the trained quantizer
    np.testing.assert_array_equal(to_np(derived), to_np(binding.derive_codebooks(cb, bbar)))
    codes = binding.encode(x, cb)
    ids, dist = binding.search(x[:16].contiguous(), cb, derived, codes, 200, 10)
    torch.cuda.synchronize()
    ref = oracle.search_flat(to_np(cb), to_np(derived), to_np(codes).astype(np.uint16), x_np[:16], 200, 10, b=b, bbar=bbar)
    np.testing.assert_allclose(to_np(dist), ref["dist"], rtol=1e-5, atol=1e-6)


def test_training_argument_errors():
    p = torch.zeros((100, 4), device=DEV)
    with pytest.raises(binding.DcpqError):
        binding.kmeans_same_size(p, p[:8].clone(), 1)            # 100 is not a multiple of 8
    with pytest.raises(binding.DcpqError):
        binding.build_quantizers(p, torch.zeros((1, 4096, 4), device=DEV), 8, 1, 1)     # b = 12
