"""nomad_pca_init against the oracle.  Eigenvectors are limits, not finite formulas: the two sides agree to the
solver's residual divided by the spectral gap, far below float32 resolution for spectra with a gap; the tolerance
is 1e-5 of the largest coordinate (float32 rounding of the scores is 6e-8 of it)."""
import numpy as np
import pytest
import torch

from oracle import pca_oracle as po
from paper_2505_15511_amd import NomadError, pca_init, workloads

pytestmark = pytest.mark.gpu


def note(msg):
    print(msg, flush=True)


def _anisotropic(n, d, seed, scales=(9.0, 4.0)):
    rng = np.random.default_rng(seed)
    s = np.ones(d)
    s[:len(scales)] = scales
    Q, _ = np.linalg.qr(rng.normal(size=(d, d)))
    return ((rng.normal(size=(n, d)) * s) @ Q.T + rng.normal(size=d) * 5.0).astype(np.float32)


def _check(X, std0=0.0, tol=1e-5):
    ref, lam_ref = po.pca_init(X, std0)
    theta, st = pca_init(X, std0, return_stats=True)
    note(f"  eigenvalues {st['eigenvalues']} residual {st['residual']:.2e} after {st['iterations']} iterations")
    assert np.allclose(st["eigenvalues"], lam_ref, rtol=1e-10)
    assert st["residual"] <= 1e-9
    assert np.abs(theta - ref).max() <= tol * np.abs(ref).max()
    return theta


@pytest.mark.parametrize("n,d,scales", [(5000, 16, (9.0, 4.0)), (3000, 130, (6.0, 3.0, 2.0)), (20000, 64, (3.0, 2.5)), (2500, 768, (8.0, 5.0)),
                                        (1000, 2, (3.0, 1.0)), (777, 5, (4.0, 2.0)), (40, 100, (9.0, 4.0)),
                                        (4000, 24, (3000.0, 40.0, 0.5)), (4000, 24, (5.0, 4.9, 4.8, 4.7, 4.6, 4.5, 4.4, 4.3, 4.2, 1.5))])
def test_scores_match_the_oracle(n, d, scales):
    note(f"pca n={n} d={d}")
    _check(_anisotropic(n, d, 10 + d, scales))


def test_mixture_data_scale_and_device_memory():
    X, _ = workloads.gmm_points(30000, 50, 10, 16.0, 5, mix="dirichlet", interleave=True)
    X = X.numpy()
    theta = _check(X, std0=1e-2)
    assert abs(theta[:, 0].astype(np.float64).std() - 1e-2) < 1e-6
    dev = pca_init(torch.from_numpy(X).cuda(), 1e-2)
    assert dev.is_cuda and np.array_equal(dev.cpu().numpy(), theta)            # deterministic, same in either memory space


def test_cross_by_hand_and_rank_deficient_data():
    # four points (+-3, 0), (0, +-1), shifted, in three dimensions: the scores are the unshifted coordinates; the
    # covariance has rank 2, below the width of the iterated block
    P = np.array([[3, 0, 0], [-3, 0, 0], [0, 1, 0], [0, -1, 0]], dtype=np.float32)
    X = P + np.array([10, -7, 2], dtype=np.float32)
    theta, st = pca_init(X, return_stats=True)
    assert np.allclose(st["eigenvalues"], [4.5, 0.5], rtol=1e-12)
    assert np.abs(theta - P[:, :2]).max() < 1e-6
    # data on a line in 40 dimensions: one non-zero eigenvalue; the first coordinate is the position along the line
    t = np.linspace(-1, 1, 500)
    L = (t[:, None] * np.arange(1, 41)[None, :]).astype(np.float32)
    theta, st = pca_init(L, return_stats=True)
    ref, lam = po.pca_init(L)
    assert abs(st["eigenvalues"][0] - lam[0]) < 1e-9 * lam[0] and abs(st["eigenvalues"][1]) < 1e-9 * lam[0]
    assert np.abs(theta[:, 0] - ref[:, 0]).max() < 1e-5 * np.abs(ref[:, 0]).max()
    assert np.abs(theta[:, 1]).max() < 1e-5 * np.abs(ref[:, 0]).max()


def test_bad_arguments():
    X = _anisotropic(100, 8, 1)
    with pytest.raises(NomadError):
        pca_init(X[:1])
    with pytest.raises(NomadError):
        pca_init(X[:, :1])
    with pytest.raises(NomadError):
        pca_init(np.zeros((50, 769), dtype=np.float32))
    with pytest.raises(NomadError):
        pca_init(np.ones((50, 4), dtype=np.float32), std0=1.0)                   # no variance to scale
