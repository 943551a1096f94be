"""Pins for the K-Means oracle: scipy's vector quantiser for the E step, closed forms for the M step, the monotone
inertia and the fixed point that Lloyd's iteration has."""
import numpy as np
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
