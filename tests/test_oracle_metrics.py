"""Pins for the oracle of the two quality measures of Section 4 (neighbourhood preservation, random triplet
accuracy): library routines (scipy's k-d tree and distance matrices), enumeration on tiny inputs, closed forms."""
import itertools

import numpy as np
import pytest
from scipy.spatial import cKDTree
from scipy.spatial.distance import cdist

from oracle import metrics_oracle as mo


def test_triplets_are_distinct_in_range_and_reproducible():
    for n in (3, 4, 7, 1000, 2**31 - 300):
        i, j, k = mo.random_triplets(n, 20000, seed=5)
        for a in (i, j, k):
            assert a.min() >= 0 and a.max() < n
        assert np.all(i != j) and np.all(i != k) and np.all(j != k)
    a = mo.random_triplets(1000, 100, seed=9, first=50)
    b = mo.random_triplets(1000, 150, seed=9)
    for x, y in zip(a, b):
        assert np.array_equal(x, y[50:])                       # triplet t depends on (t, seed) alone
    c = mo.random_triplets(1000, 150, seed=10)
    assert not np.array_equal(b[0], c[0])


def test_every_ordered_triple_is_equally_likely():
    n, T = 5, 600000
    i, j, k = mo.random_triplets(n, T, seed=11)
    counts = np.zeros((n, n, n), dtype=np.int64)
    np.add.at(counts, (i, j, k), 1)
    triples = [t for t in itertools.permutations(range(n), 3)]
    assert counts.sum() == sum(counts[t] for t in triples) == T
    expect = T / len(triples)                                  # 60 ordered triples: 10,000 each
    chi2 = sum((counts[t] - expect) ** 2 / expect for t in triples)
    assert chi2 < 59 + 6 * np.sqrt(2 * 59)                      # chi-square with 59 degrees of freedom, six sigma


def test_triplet_accuracy_closed_forms():
    rng = np.random.default_rng(0)
    X = rng.normal(size=(300, 12)).astype(np.float32)
    T = 50000
    # the same space, and a power-of-two multiple of it (exact in floating point): every triplet agrees
    assert mo.random_triplet_accuracy(X, X, T, seed=1) == (T, 1.0)
    assert mo.random_triplet_accuracy(X, 4.0 * X, T, seed=1)[0] == T
    # a projection that collapses everything: D_Y(i,j) < D_Y(i,k) is never true, so a triplet agrees iff
    # D_X(i,j) >= D_X(i,k): half of them, and exactly the complement of the swapped-roles count
    Z = np.zeros((300, 2), dtype=np.float32)
    agree, acc = mo.random_triplet_accuracy(X, Z, T, seed=1)
    i, j, k = mo.random_triplets(300, T, seed=1)
    D = cdist(X.astype(np.float64), X.astype(np.float64), "sqeuclidean")
    assert agree == int(np.count_nonzero(~(D[i, j] < D[i, k])))
    assert abs(acc - 0.5) < 4 * 0.5 / np.sqrt(T)
    # an unrelated projection: one half
    Y = rng.normal(size=(300, 2)).astype(np.float32)
    assert abs(mo.random_triplet_accuracy(X, Y, T, seed=2)[1] - 0.5) < 5 * 0.5 / np.sqrt(T)


def test_triplet_accuracy_worked_example_by_hand():
    # three points on a line at 0, 1, 3; projected to 0, 3, 1.  Squared distances: X: d01 = 1, d02 = 9, d12 = 4;
    # Y: d01 = 9, d02 = 1, d12 = 4.  For every anchor the nearer of the other two differs: no triplet agrees.
    X = np.array([[0.0], [1.0], [3.0]], dtype=np.float32)
    Y = np.array([[0.0], [3.0], [1.0]], dtype=np.float32)
    assert mo.random_triplet_accuracy(X, Y, 1000, seed=3) == (0, 0.0)
    # projected to 0, 2, 3 instead (d01 = 4, d02 = 9, d12 = 1): anchors 0 and 2 keep their nearer point (1), anchor 1's
    # moves from 0 to 2
    Y2 = np.array([[0.0], [2.0], [3.0]], dtype=np.float32)
    i, j, k = mo.random_triplets(3, 6000, seed=4)
    agree, _ = mo.random_triplet_accuracy(X, Y2, 6000, seed=4)
    assert agree == int(np.count_nonzero(i != 1))


def test_triplet_accuracy_matches_population_value_and_scipy_distances():
    rng = np.random.default_rng(7)
    n = 9
    X = rng.normal(size=(n, 5)).astype(np.float32)
    Y = (X[:, :2] + 0.8 * rng.normal(size=(n, 2))).astype(np.float32)
    DX = cdist(X.astype(np.float64), X.astype(np.float64), "sqeuclidean")
    DY = cdist(Y.astype(np.float64), Y.astype(np.float64), "sqeuclidean")
    triples = list(itertools.permutations(range(n), 3))
    population = np.mean([(DX[i, j] < DX[i, k]) == (DY[i, j] < DY[i, k]) for i, j, k in triples])
    T = 200000
    agree, acc = mo.random_triplet_accuracy(X, Y, T, seed=12, chunk=70000)      # chunking changes nothing
    assert agree == mo.random_triplet_accuracy(X, Y, T, seed=12)[0]
    assert abs(acc - population) < 5 * np.sqrt(population * (1 - population) / T)
    i, j, k = mo.random_triplets(n, T, seed=12)
    assert agree == int(np.count_nonzero((DX[i, j] < DX[i, k]) == (DY[i, j] < DY[i, k])))


def test_row_distances_follow_the_summation_order():
    # (2^26)^2 + 1 + 1 = 2^52 + 2 is exact in float64 and lost in a float32 accumulator: pins the precision
    A = np.array([[0, 0, 0], [2.0**26, 1.0, 1.0]], dtype=np.float32)
    assert mo.row_distances(A, np.array([0]), np.array([1]))[0] == 2.0**52 + 2.0
    # (2^27)^2 = 2^54 has spacing 4: added in the order t = 0, 1, 2, 3 each 1 is rounded away; any order that adds
    # the small terms first gives 2^54 + 4: pins the order
    B = np.array([[0, 0, 0, 0], [2.0**27, 1.0, 1.0, 1.0]], dtype=np.float32)
    assert mo.row_distances(B, np.array([0]), np.array([1]))[0] == 2.0**54
    assert mo.row_distances(B[:, ::-1], np.array([0]), np.array([1]))[0] == 2.0**54 + 4.0


def test_neighbours_against_scipy_kdtree():
    rng = np.random.default_rng(3)
    X = rng.normal(size=(500, 6)).astype(np.float32)
    q = np.array([0, 17, 499, 250, 17])
    got = mo.exact_neighbours(X, q, 10)
    _, idx = cKDTree(X.astype(np.float64)).query(X[q].astype(np.float64), k=11)
    assert np.array_equal(got, idx[:, 1:])


def test_neighbours_ties_duplicates_and_small_sets():
    # a square with a duplicated corner: point 0's neighbours are 4 (distance 0), then 1 and 2 (tie, lower index first)
    X = np.array([[0, 0], [1, 0], [0, 1], [1, 1], [0, 0]], dtype=np.float32)
    got = mo.exact_neighbours(X, np.arange(5), 3)
    assert got[0].tolist() == [4, 1, 2]
    assert got[4].tolist() == [0, 1, 2]
    assert got[3].tolist() == [1, 2, 0]
    assert mo.exact_neighbours(X[:3], np.arange(3), 4).tolist() == [[1, 2, -1, -1], [0, 2, -1, -1], [0, 1, -1, -1]]


def test_preservation_closed_forms():
    rng = np.random.default_rng(5)
    n, k = 400, 15
    X = rng.normal(size=(n, 8)).astype(np.float32)
    assert mo.neighbourhood_preservation(X, X, k) == (n * k, 1.0)
    assert mo.neighbourhood_preservation(X, -2.0 * X, k)[0] == n * k       # a similarity keeps every neighbourhood
    # an unrelated projection: each of the k low-dimensional neighbours is a high-dimensional one with chance k/(n-1)
    Y = rng.normal(size=(n, 2)).astype(np.float32)
    hits, value = mo.neighbourhood_preservation(X, Y, k)
    assert abs(value - k / (n - 1)) < 0.02
    # against scipy on a sample of queries
    q = rng.choice(n, 50, replace=False)
    hits, value = mo.neighbourhood_preservation(X, Y, k, q)
    _, a = cKDTree(X.astype(np.float64)).query(X[q].astype(np.float64), k=k + 1)
    _, b = cKDTree(Y.astype(np.float64)).query(Y[q].astype(np.float64), k=k + 1)
    assert hits == sum(len(set(r[1:]) & set(s[1:])) for r, s in zip(a, b))
    assert value == hits / (k * 50)


def test_preservation_by_hand():
    # five points on a line, k = 2; the projection swaps the two ends' order
    X = np.array([[0.0], [1.0], [2.1], [3.3], [4.6]], dtype=np.float32)
    Y = np.array([[4.6], [1.0], [2.1], [3.3], [0.0]], dtype=np.float32)
    # X: N(0) = {1,2} N(1) = {0,2} N(2) = {1,3} N(3) = {2,4} N(4) = {3,2}
    # Y: positions 4.6, 1, 2.1, 3.3, 0: N(0) = {3,2} N(1) = {4,2} N(2) = {1,3} N(3) = {2,0} N(4) = {1,2}
    assert mo.neighbourhood_preservation(X, Y, 2) == (1 + 1 + 2 + 1 + 1, 6 / 10)


def test_too_few_points():
    with pytest.raises(ValueError):
        mo.random_triplets(2, 10, seed=0)
