"""Pins of the oracle's training and encoding functions (Sec. 3.2, Alg. 2) against things that are not
the oracle: numpy brute force, closed forms on constructed data, scikit-learn's Lloyd iteration, a
hand-worked example, invariants the definitions imply, and the index example the paper prints."""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def blobs(rng, centres, per, sigma):
    pts = np.concatenate([c[None, :] + sigma * rng.normal(size=(per, centres.shape[1])) for c in centres])
    return pts.astype(np.float32)


# ---- assign / encode --------------------------------------------------------------------------

def test_assign_matches_numpy_bruteforce_also_on_a_strided_view():
    rng = np.random.default_rng(1)
    X = rng.normal(size=(300, 10)).astype(np.float32)
    Cb = rng.normal(size=(37, 4)).astype(np.float32)
    view = X[:, 3:7]                                          # sub-vector 3..6 of wider rows
    lab, d2 = oracle.assign(view, Cb, want_dist=True)
    full = ((view.astype(np.float64)[:, None, :] - Cb.astype(np.float64)[None, :, :]) ** 2).sum(2)
    np.testing.assert_array_equal(lab, full.argmin(1))
    np.testing.assert_allclose(d2, full.min(1), rtol=1e-14)


def test_assign_tie_goes_to_the_smaller_index():
    Cb = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 0.0], [0.0, -1.0]], np.float32)   # 0 and 2 identical
    X = np.array([[1.0, 0.0], [0.0, 0.0], [0.9, 0.1]], np.float32)                 # row 1 is equidistant from all
    np.testing.assert_array_equal(oracle.assign(X, Cb), [0, 0, 0])


def test_encode_of_decodable_vectors_returns_their_codes_and_is_nearest():
    rng = np.random.default_rng(2)
    m, kc, dsub = 3, 32, 4
    Cb = (rng.normal(size=(m, kc, dsub)) * 5).astype(np.float32)
    codes = rng.integers(0, kc, size=(50, m)).astype(np.uint16)
    X = np.concatenate([Cb[j][codes[:, j]] for j in range(m)], axis=1)
    np.testing.assert_array_equal(oracle.encode(X, Cb), codes)
    Y = (rng.normal(size=(40, m * dsub)) * 5).astype(np.float32)
    got = oracle.encode(Y, Cb)
    for j in range(m):
        full = ((Y[:, None, j * dsub:(j + 1) * dsub].astype(np.float64) - Cb[j].astype(np.float64)[None]) ** 2).sum(2)
        np.testing.assert_array_equal(got[:, j], full.argmin(1))


# ---- k-means (step 1) -------------------------------------------------------------------------

def test_kmeans_on_separated_blobs_converges_to_the_blob_means():
    rng = np.random.default_rng(3)
    centres = np.array([[0, 0], [20, 0], [0, 20], [20, 20]], np.float64)
    X = blobs(rng, centres, 50, 0.5)
    init = (centres + 2.0).astype(np.float32)                  # one initial centroid near every blob
    Cb, lab = oracle.kmeans(X, init, 5)
    np.testing.assert_array_equal(lab, np.repeat(np.arange(4), 50))
    want = X.astype(np.float64).reshape(4, 50, 2).mean(1)
    np.testing.assert_allclose(Cb, want.astype(np.float32), rtol=0, atol=1e-6)


def test_kmeans_objective_never_increases_and_labels_are_nearest_to_the_returned_centroids():
    rng = np.random.default_rng(4)
    X = rng.normal(size=(500, 6)).astype(np.float32)
    init = X[:16].copy()
    prev = np.inf
    for iters in range(0, 7):
        Cb, lab = oracle.kmeans(X, init, iters)
        obj = ((X.astype(np.float64) - Cb.astype(np.float64)[lab]) ** 2).sum()
        assert obj <= prev * (1 + 1e-12)
        prev = obj
        np.testing.assert_array_equal(lab, oracle.assign(X, Cb))
    assert prev < ((X.astype(np.float64) - init.astype(np.float64)[oracle.assign(X, init)]) ** 2).sum()


def test_kmeans_matches_scikit_learn_lloyd_from_the_same_start():
    sk = pytest.importorskip("sklearn.cluster")
    rng = np.random.default_rng(5)
    centres = rng.uniform(-30, 30, size=(12, 5))
    X = blobs(rng, centres, 40, 1.0)
    init = X[np.arange(12) * 40 + 7].copy()                    # one point of every blob
    compared = 0
    for iters in (1, 3, 8):
        Cb, lab = oracle.kmeans(X, init, iters)
        ref = sk.KMeans(n_clusters=12, init=init.astype(np.float64), n_init=1, max_iter=iters, tol=0.0,
                        algorithm="lloyd").fit(X.astype(np.float64))
        if len(np.unique(ref.labels_)) < 12 or len(np.unique(lab)) < 12:
            continue                                            # the two treat a cluster without members differently
        np.testing.assert_array_equal(lab, ref.labels_)
        np.testing.assert_allclose(Cb, ref.cluster_centers_, rtol=1e-5, atol=1e-5)
        compared += 1
    assert compared == 3


def test_kmeans_centroid_without_members_keeps_its_value():
    X = np.array([[0.0], [1.0], [2.0], [3.0]], np.float32)
    init = np.array([[1.0], [100.0]], np.float32)
    Cb, lab = oracle.kmeans(X, init, 3)
    np.testing.assert_array_equal(lab, [0, 0, 0, 0])
    np.testing.assert_array_equal(Cb, np.array([[1.5], [100.0]], np.float32))


# ---- balanced assignment / same-size k-means (step 2) -----------------------------------------

def test_balanced_assignment_hand_worked_example():
    # 4 points, 2 clusters of 2.  Round 1: points 0, 1, 2 propose to cluster 0 (their nearest), point 3 to
    # cluster 1.  Cluster 0 keeps the two closest proposers (points 1 and 0: distances 1 and 2), point 2
    # (distance 3) is turned away; cluster 1 takes point 3.  Round 2: point 2 goes to cluster 1.
    D = np.array([[2.0, 9.0], [1.0, 9.0], [3.0, 4.0], [8.0, 5.0]], np.float32)
    lab, rounds = oracle.balanced_assign(D)
    np.testing.assert_array_equal(lab, [0, 0, 1, 1])
    assert rounds == 2


def test_balanced_assignment_ties_by_point_then_cluster_index():
    D = np.ones((4, 2), np.float32)                             # all equal: everyone proposes to cluster 0
    lab, rounds = oracle.balanced_assign(D)
    np.testing.assert_array_equal(lab, [0, 0, 1, 1])            # the two smallest point indices are kept
    assert rounds == 2


def test_balanced_assignment_equals_nearest_assignment_when_that_is_balanced():
    rng = np.random.default_rng(6)
    centres = np.array([[0, 0], [50, 0], [0, 50]], np.float64)
    X = blobs(rng, centres, 8, 1.0)
    D = ((X[:, None, :].astype(np.float64) - centres[None]) ** 2).sum(2).astype(np.float32)
    lab, rounds = oracle.balanced_assign(D)
    np.testing.assert_array_equal(lab, D.argmin(1))
    assert rounds == 1


@pytest.mark.parametrize("seed,n,kbar", [(7, 64, 4), (8, 256, 16), (9, 96, 32)])
def test_balanced_assignment_sizes_and_partition(seed, n, kbar):
    rng = np.random.default_rng(seed)
    D = rng.gamma(2.0, size=(n, kbar)).astype(np.float32)
    lab, rounds = oracle.balanced_assign(D)
    assert lab.max() < kbar and rounds >= 1
    np.testing.assert_array_equal(np.bincount(lab, minlength=kbar), np.full(kbar, n // kbar))
    # a point that did not get its nearest cluster was turned away by a full one: that cluster's members
    # accepted in the round the point proposed, or before, fill it completely
    for i in np.nonzero(lab != D.argmin(1))[0]:
        assert (lab == D[i].argmin()).sum() == n // kbar
    with pytest.raises(ValueError):
        oracle.balanced_assign(D[:n - 1])


def test_same_size_kmeans_groups_are_equal_and_centroids_are_their_means():
    rng = np.random.default_rng(10)
    P = rng.normal(size=(128, 5)).astype(np.float32)
    init = P[:8].copy()
    for iters in (1, 4):
        Cbar, lab = oracle.kmeans_same_size(P, init, iters)
        np.testing.assert_array_equal(np.bincount(lab, minlength=8), np.full(8, 16))
        want = np.stack([P[lab == l].astype(np.float64).mean(0) for l in range(8)])
        np.testing.assert_allclose(Cbar, want.astype(np.float32), rtol=0, atol=1e-6)


def test_same_size_kmeans_recovers_equal_sized_blobs_where_plain_kmeans_start_is_lopsided():
    rng = np.random.default_rng(11)
    centres = np.array([[0, 0], [30, 0], [0, 30], [30, 30]], np.float64)
    P = blobs(rng, centres, 16, 1.0)
    perm = rng.permutation(len(P))
    P = P[perm]
    truth = (perm // 16).astype(np.uint32)
    init = (centres + np.array([[3, 3], [-3, 3], [3, -3], [-3, -3]])).astype(np.float32)
    Cbar, lab = oracle.kmeans_same_size(P, init, 3)
    np.testing.assert_array_equal(lab, truth)
    np.testing.assert_allclose(Cbar, np.stack([P[truth == l].astype(np.float64).mean(0) for l in range(4)]), atol=1e-5)


# ---- final codebook (step 3) ------------------------------------------------------------------

def read_golden_example():
    vals = {}
    for line in open(os.path.join(GOLDEN, "fig1c_index_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, *rest = line.split()
        vals[key] = [int(x) for x in rest]
    return vals["b"][0], vals["bbar"][0], vals["cluster"][0], vals["indexes"]


def test_final_codebook_gives_the_printed_indexes_to_the_members_of_a_cluster():
    b, bbar, cluster, indexes = read_golden_example()
    k = 1 << b
    rng = np.random.default_rng(12)
    label = np.repeat(np.arange(1 << bbar), k >> bbar).astype(np.uint32)
    label = label[rng.permutation(k)]
    Ct = rng.normal(size=(k, 3)).astype(np.float32)
    Cf, perm = oracle.build_final_codebook(Ct, label, bbar)
    got = [f for f in range(k) if label[perm[f]] == cluster]
    assert sorted(got) == sorted(indexes)


def test_final_codebook_property_p1_and_order_inside_a_group():
    rng = np.random.default_rng(13)
    b, bbar, d = 8, 3, 4
    k, kbar = 1 << b, 1 << bbar
    label = np.repeat(np.arange(kbar), k // kbar).astype(np.uint32)[rng.permutation(k)]
    Ct = rng.normal(size=(k, d)).astype(np.float32)
    Cf, perm = oracle.build_final_codebook(Ct, label, bbar)
    assert sorted(perm.tolist()) == list(range(k))
    np.testing.assert_array_equal(Cf, Ct[perm])
    f = np.arange(k)
    np.testing.assert_array_equal(label[perm], f & (kbar - 1))               # P1: low bits = group
    for l in range(kbar):
        members = perm[(f & (kbar - 1)) == l]                                # in increasing final index
        assert (np.diff(members.astype(np.int64)) > 0).all()                 # = increasing temporary index
    # the derived codebook of the final codebook is the mean of every group
    der = oracle.derive_codebooks(Cf[None], b=b, bbar=bbar)[0]
    want = np.stack([Ct[label == l].astype(np.float64).mean(0) for l in range(kbar)])
    np.testing.assert_allclose(der, want, rtol=1e-5, atol=1e-6)
    with pytest.raises(ValueError):
        oracle.build_final_codebook(Ct, np.zeros(k, np.uint32), bbar)


def test_alg2_end_to_end_derived_codebook_equals_the_same_size_centroids():
    rng = np.random.default_rng(14)
    b, bbar, d = 6, 2, 3
    X = rng.normal(size=(2000, d)).astype(np.float32)
    Ct, _ = oracle.kmeans(X, X[:1 << b].copy(), 4)
    Cbar, lab = oracle.kmeans_same_size(Ct, Ct[:1 << bbar].copy(), 3)
    Cf, perm = oracle.build_final_codebook(Ct, lab, bbar)
    der = oracle.derive_codebooks(Cf[None], b=b, bbar=bbar)[0]
    np.testing.assert_allclose(der, Cbar, rtol=1e-5, atol=1e-6)
    # encoding with the final codebook: the low bits of a code name the group of the centroid it picked
    codes = oracle.encode(X[:200], Cf[None])
    np.testing.assert_array_equal(codes[:, 0] & ((1 << bbar) - 1), lab[perm[codes[:, 0]]])
