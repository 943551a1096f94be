"""Pins for the K-Means oracle: scipy's vector quantiser for the E step, closed forms for the M step, the monotone
inertia and the fixed point that Lloyd's iteration has."""
import numpy as np
import pytest
from scipy.cluster.vq import vq

from oracle import kmeans_oracle as km


def test_assignment_agrees_with_scipy_vq():
    rng = np.random.default_rng(1)
    X = rng.normal(size=(2000, 9)).astype(np.float32)
    C = rng.normal(size=(17, 9)).astype(np.float32)
    labels, dist = km.assign(X, C)
    code, d = vq(X.astype(np.float64), C.astype(np.float64))
    assert np.array_equal(labels, code) and np.allclose(dist, d ** 2, rtol=1e-12)


def test_ties_go_to_the_lower_centroid():
    X = np.array([[0.0, 0.0], [1.0, 0.0], [0.5, 7.0]], dtype=np.float32)
    C = np.array([[1.0, 0.0], [-1.0, 0.0], [1.0, 0.0], [0.0, 1.0], [0.0, -1.0]], dtype=np.float32)
    labels, dist = km.assign(X, C)
    assert labels.tolist() == [0, 0, 3] and dist.tolist() == [1.0, 0.0, 36.25]


def test_update_is_the_mean_and_empty_clusters_keep_their_centroid():
    X = np.array([[1, 2], [3, 4], [5, 6], [10, 10]], dtype=np.float32)
    C_old = np.array([[9, 9], [8, 8], [7, 7]], dtype=np.float32)
    C = km.update(X, np.array([0, 0, 0, 2]), C_old)
    assert C.tolist() == [[3.0, 4.0], [8.0, 8.0], [10.0, 10.0]]
    rng = np.random.default_rng(2)
    X = rng.normal(size=(500, 4)).astype(np.float32)
    lab = rng.integers(0, 6, 500)
    C = km.update(X, lab, np.zeros((6, 4), np.float32))
    for j in range(6):
        assert np.allclose(C[j], X[lab == j].astype(np.float64).mean(0), rtol=1e-6)


def test_inertia_never_rises_and_the_result_is_a_fixed_point():
    rng = np.random.default_rng(3)
    X = np.concatenate([rng.normal(size=(300, 5)) + 6 * rng.normal(size=(1, 5)) for _ in range(6)]).astype(np.float32)
    C0 = X[rng.choice(len(X), 6, replace=False)]
    inertias = []
    C = C0
    for it in range(1, 30):
        C, labels, ran, inertia = km.lloyd(X, C0, it)
        inertias.append(inertia)
        if ran < it:
            break
    assert all(b <= a + 1e-9 for a, b in zip(inertias, inertias[1:]))
    assert ran < 29                                                        # converged
    lab2, _ = km.assign(X, C)
    assert np.array_equal(lab2, labels) and np.array_equal(km.update(X, labels, C), C)


def test_well_separated_blobs_are_recovered():
    rng = np.random.default_rng(4)
    centres = np.array([[0, 0], [20, 0], [0, 20], [20, 20]], dtype=np.float64)
    truth = rng.integers(0, 4, 800)
    X = (centres[truth] + rng.normal(size=(800, 2))).astype(np.float32)
    C, labels, ran, _ = km.lloyd(X, (centres + 3.0).astype(np.float32), 50)
    assert np.array_equal(labels, truth) and np.abs(C - centres).max() < 0.3 and ran <= 4


# ---------------------------------------------------------------- the start from a locality-sensitive hash
def _hash_inputs(n, d, b, seed):
    rng = np.random.default_rng(seed)
    X = rng.normal(size=(n, d)).astype(np.float32)
    return X, rng.normal(size=(b, d)).astype(np.float32), rng.choice(n, b, replace=False)


def test_hash_bits_against_a_matrix_product():
    X, planes, anchors = _hash_inputs(4000, 24, 5, 1)
    proj = (X.astype(np.float64)[:, None, :] - X.astype(np.float64)[anchors][None, :, :]) * planes.astype(np.float64)[None, :, :]
    proj = proj.sum(axis=2)                                                  # another summation order: compare away from 0
    code = ((proj > 0) * (1 << np.arange(5))).sum(axis=1)
    clear = (np.abs(proj) > 1e-9).all(axis=1)
    got = km.lsh_buckets(X, planes, anchors, 32)                             # K = 2^b: the bucket is the code
    assert clear.mean() > 0.99 and np.array_equal(got[clear], code[clear])
    for K in (7, 20, 31):
        assert np.array_equal(km.lsh_buckets(X, planes, anchors, K)[clear], (code[clear] * K) // 32)
    with pytest.raises(ValueError):
        km.lsh_buckets(X, planes, anchors, 33)


def test_hash_sides_known_by_construction():
    # plane 0: normal e_0 through point 2 (x_0 = 1): bit 0 = [x_0 > 1]; plane 1: normal -e_1 through point 0 (x_1 = 0): bit 1 = [x_1 < 0]
    X = np.array([[0, 0], [2, 0], [1, 5], [3, -1], [1, -2], [-4, -4]], dtype=np.float32)
    planes = np.array([[1, 0], [0, -1]], dtype=np.float32)
    buckets = km.lsh_buckets(X, planes, np.array([2, 0]), 4)
    assert buckets.tolist() == [0, 1, 0, 3, 2, 2]        # a point on a plane (the anchors, and point 4 on plane 0) gets bit 0
    C, _ = km.lsh_init(X, planes, np.array([2, 0]), 4)
    assert np.array_equal(C, np.array([[0.5, 2.5], [2, 0], [-1.5, -3], [3, -1]], dtype=np.float32))
    # three buckets from two planes: codes 0, 1 -> bucket 0, code 2 -> 1, code 3 -> 2
    assert km.lsh_buckets(X, planes, np.array([2, 0]), 3).tolist() == [0, 0, 0, 2, 1, 1]


def test_hash_start_means_and_empty_buckets():
    X, planes, anchors = _hash_inputs(3000, 10, 4, 2)
    C, buckets = km.lsh_init(X, planes, anchors, 16)
    for j in range(16):
        members = X[buckets == j].astype(np.float64)
        if len(members):
            assert np.allclose(C[j], members.mean(axis=0), rtol=0, atol=1e-6)
        else:
            assert np.array_equal(C[j], X[j * 3000 // 16])
    assert len(np.unique(buckets)) >= 8
    # every point on one side of the single plane used twice: buckets 1 and 2 of 4 are empty and take points n/4, n/2
    Y = np.abs(X) + 1.0
    Y[0] = 0.0
    planes2 = np.ones((2, 10), dtype=np.float32)
    C, buckets = km.lsh_init(Y, planes2, np.array([0, 0]), 4)
    assert set(buckets.tolist()) == {0, 3} and np.count_nonzero(buckets == 0) == 1
    assert np.array_equal(C[1], Y[750]) and np.array_equal(C[2], Y[1500]) and np.array_equal(C[0], Y[0])
    # a start from the hash is a valid start: Lloyd's iterations lower the inertia from it
    X3 = np.concatenate([X + 6.0, X - 6.0]).astype(np.float32)
    C0, _ = km.lsh_init(X3, planes, anchors, 16)
    _, d0 = km.assign(X3, C0)
    _, _, _, inertia = km.lloyd(X3, C0, 10)
    assert inertia < d0.sum()


def test_median_anchors_split_the_data_in_halves():
    rng = np.random.default_rng(8)
    X = (rng.normal(size=(5000, 12)) * rng.uniform(0.5, 3.0, size=12) + rng.normal(size=12) * 4).astype(np.float32)
    planes = rng.normal(size=(6, 12)).astype(np.float32)
    anchors = km.lsh_median_anchors(X, planes)
    idx = (np.arange(1024) * 5000) // 1024
    proj = X[idx].astype(np.float64) @ planes.astype(np.float64).T            # library route: the sample's projections
    for j in range(6):
        assert anchors[j] in idx
        below = np.count_nonzero(proj[:, j] < proj[np.nonzero(idx == anchors[j])[0][0], j])
        assert below == 512                                                   # rank m / 2 of 1024 distinct values
    buckets = km.lsh_buckets(X, planes, anchors, 64)
    bits = np.stack([(buckets >> j) & 1 for j in range(6)], axis=1)            # K = 2^b: the bucket is the code
    assert np.abs(bits.mean(axis=0) - 0.5).max() < 0.05                        # every plane halves the data
    counts = np.bincount(buckets, minlength=64)
    assert counts.max() < 6 * 5000 / 64                                        # no giant bucket (planes through far points leave some)


def test_median_anchor_by_hand_and_small_inputs():
    # five points on a line, normal +e_0: projections 3, 1, 4, 1, 5 -> ascending (projection, index): 1, 3, 0, 2, 4; rank 2 = point 0
    X = np.array([[3, 0], [1, 0], [4, 0], [1, 0], [5, 0]], dtype=np.float32)
    assert km.lsh_median_anchors(X, np.array([[1, 0]], dtype=np.float32)).tolist() == [0]
    assert km.lsh_median_anchors(X, np.array([[-1, 0]], dtype=np.float32)).tolist() == [0]      # -5 -4 -3 -1 -1: rank 2 = point 0
    assert km.lsh_median_anchors(X, np.array([[0, 1]], dtype=np.float32)).tolist() == [2]       # all ties: by index
    assert km.lsh_median_anchors(X[:1], np.array([[1, 0]], dtype=np.float32)).tolist() == [0]
