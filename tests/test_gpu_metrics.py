"""The two quality measures of Section 4 on the GPU against the oracle: both are counts of exact decisions, so they
must agree to the last unit."""
import numpy as np
import pytest
import torch

from oracle import metrics_oracle as mo
from paper_2505_15511_amd import NomadError, neighbourhood_preservation, random_triplet_accuracy, workloads

pytestmark = pytest.mark.gpu


def note(msg):
    print(msg, flush=True)


def _spaces(n, d, d_low, seed, noise=0.5):
    X, _ = workloads.gmm_points(n, d, 8, 16.0, seed, mix="dirichlet", interleave=True)
    X = X.numpy()
    rng = np.random.default_rng(seed)
    Y = (X[:, :d_low] + noise * rng.normal(size=(n, d_low))).astype(np.float32)    # a noisy linear projection
    return X, Y


@pytest.mark.parametrize("n,d,d_low,T", [(3000, 50, 2, 200000), (500, 7, 3, 70001), (4000, 768, 2, 50000), (3, 4, 1, 1000), (2000, 128, 2, 0)])
def test_triplet_accuracy_matches_the_oracle_exactly(n, d, d_low, T):
    note(f"triplets n={n} d={d} d_low={d_low} T={T}")
    X, Y = _spaces(n, d, d_low, 40 + d)
    ref = mo.random_triplet_accuracy(X, Y, T, seed=77)[0] if T else 0                   # no triplets: nothing agrees
    agree, acc = random_triplet_accuracy(X, Y, T, 77)                                   # host arrays
    assert agree == ref
    agree_dev, _ = random_triplet_accuracy(torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda(), T, 77)
    assert agree_dev == ref
    if T:
        assert acc == ref / T


def test_triplet_accuracy_special_cases():
    X, Y = _spaces(2000, 32, 2, 5)
    assert random_triplet_accuracy(X, X, 100000, 1)[0] == 100000                        # the same space
    agree, _ = random_triplet_accuracy(X, np.zeros_like(Y), 100000, 1)                  # a collapsed projection
    assert agree == mo.random_triplet_accuracy(X, np.zeros_like(Y), 100000, 1)[0]
    a = random_triplet_accuracy(X, Y, 100000, (5 << 32) | 9)[0]                         # both key words are used
    assert a == mo.random_triplet_accuracy(X, Y, 100000, (5 << 32) | 9)[0]
    assert a != random_triplet_accuracy(X, Y, 100000, 9)[0]
    # duplicates and exact ties: integer grid
    G = np.random.default_rng(3).integers(0, 3, size=(500, 6)).astype(np.float32)
    H = G[:, :2].copy()
    assert random_triplet_accuracy(G, H, 50000, 2)[0] == mo.random_triplet_accuracy(G, H, 50000, 2)[0]


def test_triplet_accuracy_at_large_triplet_counts():
    # triplet t depends on (t, seed) alone: a run and a slightly longer one differ by exactly the tail's triplets
    X, Y = _spaces(100000, 16, 2, 8)
    Xd, Yd = torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda()
    T1, T2 = 1 << 20, (1 << 20) + 4097
    a1, a2 = random_triplet_accuracy(Xd, Yd, T1, 3)[0], random_triplet_accuracy(Xd, Yd, T2, 3)[0]
    i, j, k = mo.random_triplets(len(X), T2 - T1, 3, first=T1)
    tail = np.count_nonzero((mo.row_distances(X, i, j) < mo.row_distances(X, i, k)) == (mo.row_distances(Y, i, j) < mo.row_distances(Y, i, k)))
    assert a2 - a1 == tail


@pytest.mark.parametrize("n,d,d_low,k,nq", [(3000, 50, 2, 15, None), (5000, 16, 2, 15, 400), (2500, 200, 3, 32, 300), (1500, 7, 2, 1, None),
                                            (20, 5, 2, 15, None), (12, 3, 2, 15, 5)])
def test_neighbourhood_preservation_matches_the_oracle_exactly(n, d, d_low, k, nq):
    note(f"preservation n={n} d={d} d_low={d_low} k={k} queries={nq}")
    X, Y = _spaces(n, d, d_low, 60 + d, noise=1.5)
    q = None if nq is None else np.random.default_rng(n).choice(n, nq, replace=nq > n).astype(np.int32)
    ref_hits, ref_value = mo.neighbourhood_preservation(X, Y, k, q)
    hits, value = neighbourhood_preservation(X, Y, k, q)
    assert hits == ref_hits and value == ref_value
    qd = None if q is None else torch.from_numpy(q).cuda()
    assert neighbourhood_preservation(torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda(), k, qd)[0] == ref_hits


def test_neighbourhood_preservation_special_cases():
    X, Y = _spaces(2000, 24, 2, 9)
    assert neighbourhood_preservation(X, X, 15) == (2000 * 15, 1.0)
    # ties and duplicates in both spaces: integer grids, most queries go through the exact fallback
    G = np.random.default_rng(4).integers(0, 4, size=(600, 5)).astype(np.float32)
    H = G[:, :2].copy()
    assert neighbourhood_preservation(G, H, 10)[0] == mo.neighbourhood_preservation(G, H, 10)[0]
    # repeated queries count as often as listed
    q = np.array([5, 5, 5, 17], dtype=np.int32)
    assert neighbourhood_preservation(X, Y, 15, q)[0] == mo.neighbourhood_preservation(X, Y, 15, q)[0]


def test_bad_arguments():
    X, Y = _spaces(100, 8, 2, 1)
    with pytest.raises(NomadError):
        neighbourhood_preservation(X, Y, 33)
    with pytest.raises(NomadError):
        neighbourhood_preservation(X, Y, 5, np.array([0, 100], dtype=np.int32))
    with pytest.raises(NomadError):
        random_triplet_accuracy(X[:2], Y[:2], 10, 0)
    with pytest.raises(ValueError):
        random_triplet_accuracy(X, Y[:50], 10, 0)
