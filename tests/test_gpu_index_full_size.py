"""The index, the PCA start and the quality measures at the sizes bench.py times (n = 1e6, d = 128), against oracle
values on samples of the outputs that the oracle can compute one by one, plus properties that hold at any size."""
import numpy as np
import pytest
import torch

from oracle import kmeans_oracle as km
from oracle import knn_oracle as ko
from oracle import metrics_oracle as mo
from oracle import pca_oracle as po
from paper_2505_15511_amd import (kmeans_lloyd, knn_in_clusters, neighbourhood_preservation, pca_init, random_triplet_accuracy,
                                  workloads)

pytestmark = pytest.mark.gpu

N, D, R, K = 1_000_000, 128, 256, 15


def note(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module")
def data():
    X, c = workloads.gmm_points(N, D, R, 16.0, 4242, mix="equal", interleave=True)     # bench.py --index knn's input
    return X, c


def test_knn_at_bench_size_sampled_queries(data):
    X, c = data
    note("knn n=1e6 d=128 256 clusters k=15")
    nb = knn_in_clusters(X.cuda(), c.cuda(), R, K).cpu().numpy()
    Xn, cn = X.numpy(), c.numpy()
    assert (nb >= 0).all() and (nb < N).all()
    assert (cn[nb] == cn[:, None]).all()                                    # neighbours stay inside the cluster
    assert (nb != np.arange(N)[:, None]).all()                              # nobody is their own neighbour
    srt = np.sort(nb, axis=1)
    assert (srt[:, 1:] != srt[:, :-1]).all()                                # no neighbour twice
    rng = np.random.default_rng(0)
    for q in rng.choice(N, 300, replace=False):
        members = np.nonzero(cn == cn[q])[0]
        Dq = ko.pair_distances(Xn[q:q + 1], Xn[members])[0]
        Dq[members == q] = np.inf
        order = np.lexsort((members, Dq))[:K]
        assert np.array_equal(nb[q], members[order]), f"query {q}"


def test_kmeans_iteration_at_bench_size_sampled_labels(data):
    X, _ = data
    note("kmeans n=1e6 d=128 K=256, one iteration")
    Xn = X.numpy()
    C0 = Xn[np.random.default_rng(1).choice(N, R, replace=False)].copy()
    C, lab, it, inertia = kmeans_lloyd(X.cuda(), torch.from_numpy(C0).cuda(), 1)
    lab = lab.cpu().numpy()
    q = np.random.default_rng(2).choice(N, 20000, replace=False)
    lab_ref, dist_ref = km.assign(Xn[q], C0)
    assert np.array_equal(lab[q].astype(np.int64), lab_ref)
    assert lab.min() >= 0 and lab.max() < R and it == 1
    assert abs(inertia / N - dist_ref.mean()) < 0.02 * dist_ref.mean()       # the sample's mean distance estimates the whole
    # the new centroids are means of their clusters: their count-weighted mean is the mean of the data
    counts = np.bincount(lab, minlength=R).astype(np.float64)
    Cn = C.cpu().numpy().astype(np.float64)
    assert np.abs((Cn * counts[:, None]).sum(axis=0) / N - Xn.astype(np.float64).mean(axis=0)).max() < 1e-5


def test_pca_at_bench_size(data):
    X, _ = data
    note("pca n=1e6 d=128")
    ref, lam = po.pca_init(X.numpy(), 0.01)
    theta, st = pca_init(X.cuda(), 0.01, return_stats=True)
    note(f"  eigenvalues {st['eigenvalues']} (oracle {lam}), residual {st['residual']:.1e}, {st['iterations']} steps")
    assert np.allclose(st["eigenvalues"], lam, rtol=1e-9)
    # 256 equal components in 128 dimensions: a flat spectrum (gap 2 % of lambda_1); residual / gap bounds the axes' error
    gap = (lam[0] - lam[1]) / lam[0]
    assert np.abs(theta.cpu().numpy() - ref).max() <= max(1e-5, 20 * st["residual"] / gap) * np.abs(ref).max()


def test_quality_measures_at_bench_size(data):
    X, _ = data
    Xn = X.numpy()
    Y = (Xn[:, :2] + 0.5 * np.random.default_rng(3).normal(size=(N, 2))).astype(np.float32)
    note("triplets n=1e6 d=128 T=1e6")
    T = 1_000_000
    agree, _ = random_triplet_accuracy(X.cuda(), torch.from_numpy(Y).cuda(), T, 9)
    assert agree == mo.random_triplet_accuracy(Xn, Y, T, 9)[0]
    note("preservation n=3e5 d=128, 40 queries")
    n2 = 300_000
    q = np.random.default_rng(4).choice(n2, 40, replace=False).astype(np.int32)
    hits, _ = neighbourhood_preservation(X[:n2].cuda(), torch.from_numpy(Y[:n2]).cuda(), K, torch.from_numpy(q).cuda())
    assert hits == mo.neighbourhood_preservation(Xn[:n2], Y[:n2], K, q)[0]
