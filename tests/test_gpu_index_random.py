"""Random shapes for the index and the quality measures against their oracles: every result is a set of exact
decisions, so it must match to the last unit.  NOMAD_RANDOM_CASES_FROM / _TO widen the seed range."""
import os

import numpy as np
import pytest

from oracle import kmeans_oracle as km
from oracle import knn_oracle as ko
from oracle import metrics_oracle as mo
from paper_2505_15511_amd import (kmeans_lloyd, kmeans_lsh_init, knn_in_clusters, neighbourhood_preservation,
                                  random_triplet_accuracy)

pytestmark = pytest.mark.gpu

SEEDS = range(int(os.environ.get("NOMAD_RANDOM_CASES_FROM", 0)), int(os.environ.get("NOMAD_RANDOM_CASES_TO", 12)))


def _case(seed):
    rng = np.random.default_rng(7000 + seed)
    n = int(rng.integers(40, 3000))
    d = int(rng.choice([1, 2, 3, 5, 8, 17, 32, 33, 64, 100, 129, 200, 260, 400, 520]))
    comps = int(rng.integers(1, 9))
    kind = int(rng.integers(0, 3))
    if kind == 0:                                            # clustered, continuous
        means = rng.normal(size=(comps, d)) * 4
        lab = rng.integers(0, comps, size=n)
        X = means[lab] + rng.normal(size=(n, d))
    elif kind == 1:                                          # a coarse integer grid: ties and duplicates everywhere
        X = rng.integers(0, 3, size=(n, d)).astype(np.float64)
        lab = rng.integers(0, comps, size=n)
    else:                                                    # far from the origin, small spread
        X = 1000.0 + rng.normal(size=(n, d)) * 0.5
        lab = rng.integers(0, comps, size=n)
    return rng, X.astype(np.float32), lab.astype(np.int32), comps


@pytest.mark.parametrize("seed", SEEDS)
def test_random_index_case(seed):
    rng, X, lab, comps = _case(seed)
    n, d = X.shape
    k = int(rng.integers(1, 33))
    print(f"seed {seed}: n={n} d={d} clusters={comps} k={k}", flush=True)
    ref, _ = ko.in_cluster_knn(X, lab, k)
    assert np.array_equal(knn_in_clusters(X, lab, comps, k).astype(np.int64), ref)
    # K-Means: hash start with library anchors, then two of Lloyd's iterations
    K = int(rng.integers(1, min(n, 40) + 1))
    b = max(1, int(np.ceil(np.log2(K))))
    planes = rng.normal(size=(b, d)).astype(np.float32)
    C0_ref, buckets_ref = km.lsh_init(X, planes, km.lsh_median_anchors(X, planes), K)
    C0, buckets = kmeans_lsh_init(X, K, planes, None, return_buckets=True)
    assert np.array_equal(buckets.astype(np.int64), buckets_ref) and np.array_equal(C0, C0_ref)
    C_ref, lab_ref, it_ref, _ = km.lloyd(X, C0_ref, 2)
    C, labels, it, _ = kmeans_lloyd(X, C0, 2)
    assert it == it_ref and np.array_equal(labels.astype(np.int64), lab_ref) and np.array_equal(C, C_ref)
    # the quality measures against a noisy low-dimensional copy
    d_low = int(rng.integers(1, 4))
    Y = (X[:, :d_low] if d >= d_low else np.repeat(X, d_low, axis=1)[:, :d_low]) + rng.normal(size=(n, d_low)).astype(np.float32)
    Y = Y.astype(np.float32)
    T = int(rng.integers(1, 20000))
    if n >= 3:
        assert random_triplet_accuracy(X, Y, T, seed)[0] == mo.random_triplet_accuracy(X, Y, T, seed)[0]
    kq = int(rng.integers(1, 33))
    q = rng.choice(n, min(n, 60), replace=False).astype(np.int32) if seed % 2 else None
    if q is not None or n <= 1200:
        assert neighbourhood_preservation(X, Y, kq, q)[0] == mo.neighbourhood_preservation(X, Y, kq, q)[0]


@pytest.mark.parametrize("seed", SEEDS)
def test_random_pca_case(seed):
    from oracle import pca_oracle as po
    from paper_2505_15511_amd import pca_init
    rng = np.random.default_rng(9000 + seed)
    n = int(rng.integers(50, 5000))
    d = int(rng.choice([2, 3, 5, 8, 17, 32, 64, 100, 129, 260, 400, 768]))
    scales = np.sort(rng.uniform(0.2, 6.0, size=d))[::-1]
    Q, _ = np.linalg.qr(rng.normal(size=(d, d)))
    X = ((rng.normal(size=(n, d)) * scales) @ Q.T + rng.normal(size=d) * 10.0).astype(np.float32)
    _, lam3, _ = po.principal_axes(X, min(3, d))
    gaps = [(lam3[0] - lam3[1]) / lam3[0]] + ([(lam3[1] - lam3[2]) / lam3[0]] if d > 2 else [])
    std0 = float(rng.choice([0.0, 0.01]))
    ref, lam = po.pca_init(X, std0)
    theta, st = pca_init(X, std0, return_stats=True)
    print(f"seed {seed}: n={n} d={d} gaps {min(gaps):.3f} residual {st['residual']:.1e} after {st['iterations']}", flush=True)
    assert np.allclose(st["eigenvalues"], lam, rtol=1e-9)
    if min(gaps) > 0.01:                                     # the axes are well defined: the scores must agree
        assert np.abs(theta - ref).max() <= 1e-5 * np.abs(ref).max()
