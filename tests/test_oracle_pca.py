"""Pins for the oracle of the PCA initialisation (Section 3.5): scikit-learn's PCA, the singular value decomposition,
planted axes, an example by hand, invariances."""
import numpy as np
import pytest
from sklearn.decomposition import PCA

from oracle import pca_oracle as po


def _anisotropic(n, d, seed, scales=(9.0, 4.0)):
    rng = np.random.default_rng(seed)
    s = np.ones(d)
    s[:len(scales)] = scales
    Q, _ = np.linalg.qr(rng.normal(size=(d, d)))
    X = (rng.normal(size=(n, d)) * s) @ Q.T + rng.normal(size=d) * 5.0
    return X.astype(np.float32), Q


def _same_up_to_sign(a, b, tol):
    for c in range(a.shape[1]):
        assert min(np.abs(a[:, c] - b[:, c]).max(), np.abs(a[:, c] + b[:, c]).max()) <= tol


def test_against_scikit_learn():
    X, _ = _anisotropic(3000, 20, 1)
    theta, lam = po.pca_init(X)
    ref = PCA(n_components=2, svd_solver="full").fit(X.astype(np.float64))
    _same_up_to_sign(theta, ref.transform(X.astype(np.float64)), 2e-5)
    assert np.allclose(lam, ref.explained_variance_ * (len(X) - 1) / len(X), rtol=1e-10)    # theirs divides by n - 1


def test_against_the_singular_value_decomposition():
    X, _ = _anisotropic(500, 12, 2, scales=(5.0, 3.0, 2.0))
    mean, lam, axes = po.principal_axes(X, 3)
    Xc = X.astype(np.float64) - X.astype(np.float64).mean(axis=0)
    U, S, Vt = np.linalg.svd(Xc, full_matrices=False)
    assert np.allclose(lam, S[:3] ** 2 / len(X), rtol=1e-10)
    _same_up_to_sign(axes, Vt[:3].T, 1e-9)
    assert np.allclose(mean, X.astype(np.float64).mean(axis=0), rtol=0, atol=1e-12)


def test_planted_axes_are_recovered():
    X, Q = _anisotropic(200000, 8, 3, scales=(10.0, 3.0))
    _, lam, axes = po.principal_axes(X)
    assert abs(abs(axes[:, 0] @ Q[:, 0]) - 1) < 1e-3 and abs(abs(axes[:, 1] @ Q[:, 1]) - 1) < 1e-3
    assert abs(lam[0] - 100.0) < 2.0 and abs(lam[1] - 9.0) < 0.3


def test_cross_by_hand():
    # four points (+-3, 0), (0, +-1) shifted by (10, -7), embedded in three dimensions: mean = the shift, C = diag(4.5,
    # 0.5, 0); axes e_1, e_2; scores = the unshifted coordinates
    P = np.array([[3, 0, 0], [-3, 0, 0], [0, 1, 0], [0, -1, 0]], dtype=np.float32)
    X = P + np.array([10, -7, 2], dtype=np.float32)
    theta, lam = po.pca_init(X)
    assert np.allclose(lam, [4.5, 0.5], rtol=0, atol=1e-12)
    assert np.array_equal(theta, P[:, :2])
    # with std0 the first coordinate gets that standard deviation and the second keeps the ratio
    theta, _ = po.pca_init(X, std0=0.01)
    assert np.allclose(theta.astype(np.float64).std(axis=0), [0.01, 0.01 / 3], rtol=1e-6)
    assert np.allclose(theta, P[:, :2] * (0.01 / np.sqrt(4.5)), rtol=1e-6)


def test_orientation_rule():
    assert np.array_equal(po.orient(np.array([0.1, -0.9, 0.3])), [-0.1, 0.9, -0.3])
    assert np.array_equal(po.orient(np.array([0.5, -0.5])), [0.5, -0.5])          # equal magnitudes: the first decides
    assert np.array_equal(po.orient(np.array([-0.5, 0.5])), [0.5, -0.5])
    X, _ = _anisotropic(400, 6, 4)
    _, _, axes = po.principal_axes(X)
    for c in range(2):
        assert axes[np.argmax(np.abs(axes[:, c])), c] > 0
        assert abs(np.linalg.norm(axes[:, c]) - 1) < 1e-12
    assert abs(axes[:, 0] @ axes[:, 1]) < 1e-12


def test_invariances():
    X, _ = _anisotropic(1000, 10, 5)
    theta, lam = po.pca_init(X)
    # scores are centred and uncorrelated, with the eigenvalues as variances
    t = theta.astype(np.float64)
    assert np.abs(t.mean(axis=0)).max() < 1e-5
    assert np.allclose((t * t).mean(axis=0), lam, rtol=1e-5)
    assert abs((t[:, 0] * t[:, 1]).mean()) < 1e-4
    # a translation by exactly representable amounts changes nothing; a permutation of the points permutes the rows
    shifted, _ = po.pca_init((X.astype(np.float64) + 64.0).astype(np.float32))
    assert np.abs(shifted - theta).max() < 2e-4
    perm = np.random.default_rng(0).permutation(len(X))
    assert np.abs(po.pca_init(X[perm])[0] - theta[perm]).max() < 1e-5
    # std0 only rescales
    scaled, _ = po.pca_init(X, std0=1e-4)
    assert np.allclose(scaled, theta * (1e-4 / np.sqrt(lam[0])), rtol=1e-6, atol=1e-12)
