"""Pins for the in-cluster nearest-neighbour oracle: scipy's k-d tree run per cluster (a library routine for the same
textbook problem), hand-made examples whose neighbours can be read off, ties and duplicates, small clusters."""
import numpy as np
from scipy.spatial import cKDTree

from oracle import knn_oracle as ko


def test_points_on_a_line_have_the_neighbours_one_can_read_off():
    # cluster 0: 0, 1, 3, 7, 15 on the x axis; cluster 1: three points on the y axis
    X = np.array([[0, 0], [1, 0], [3, 0], [7, 0], [15, 0], [0, 10], [0, 11], [0, 13]], dtype=np.float32)
    c = np.array([0, 0, 0, 0, 0, 1, 1, 1])
    nb, ds = ko.in_cluster_knn(X, c, 2)
    assert nb.tolist() == [[1, 2], [0, 2], [1, 0], [2, 1], [3, 2], [6, 7], [5, 7], [6, 5]]
    assert ds[0].tolist() == [1.0, 9.0] and ds[4].tolist() == [64.0, 144.0] and ds[7].tolist() == [4.0, 9.0]


def test_neighbours_never_leave_the_cluster_and_exclude_the_point_itself():
    rng = np.random.default_rng(1)
    X = rng.normal(size=(300, 5)).astype(np.float32)
    c = rng.integers(0, 4, 300)
    nb, _ = ko.in_cluster_knn(X, c, 7)
    assert (c[nb] == c[:, None]).all() and (nb != np.arange(300)[:, None]).all()
    assert all(len(set(row)) == 7 for row in nb.tolist())


def test_agrees_with_a_kd_tree_built_per_cluster():
    rng = np.random.default_rng(2)
    n, d, k = 1500, 6, 10
    X = rng.normal(size=(n, d)).astype(np.float32)
    c = rng.integers(0, 5, n)
    nb, ds = ko.in_cluster_knn(X, c, k)
    for r in range(5):
        members = np.nonzero(c == r)[0]
        dist, idx = cKDTree(X[members].astype(np.float64)).query(X[members].astype(np.float64), k=k + 1)
        assert np.array_equal(members[idx[:, 1:]], nb[members])           # column 0 is the point itself
        assert np.allclose(dist[:, 1:] ** 2, ds[members], rtol=1e-12, atol=0)


def test_ties_go_to_the_lower_index_and_duplicates_are_ordinary_points():
    # a unit square: every corner has two neighbours at distance 1 and one at distance 2; a duplicate of corner 0
    X = np.array([[0, 0], [1, 0], [0, 1], [1, 1], [0, 0]], dtype=np.float32)
    nb, ds = ko.in_cluster_knn(X, np.zeros(5, int), 3)
    assert nb[0].tolist() == [4, 1, 2] and ds[0].tolist() == [0.0, 1.0, 1.0]
    assert nb[3].tolist() == [1, 2, 0] and ds[3].tolist() == [1.0, 1.0, 2.0]
    assert nb[4].tolist() == [0, 1, 2]


def test_small_clusters_leave_empty_slots():
    X = np.arange(12, dtype=np.float32).reshape(6, 2)
    nb, ds = ko.in_cluster_knn(X, np.array([0, 0, 0, 1, 2, 2]), 3)
    assert nb.tolist() == [[1, 2, -1], [0, 2, -1], [1, 0, -1], [-1, -1, -1], [5, -1, -1], [4, -1, -1]]
    assert np.isinf(ds[3]).all() and np.isinf(ds[0, 2])


def test_distance_is_accumulated_dimension_by_dimension_in_float64():
    rng = np.random.default_rng(3)
    a, b = rng.normal(size=(1, 40)).astype(np.float32), rng.normal(size=(1, 40)).astype(np.float32)
    acc = 0.0
    for t in range(40):
        diff = float(a[0, t]) - float(b[0, t])
        acc = acc + diff * diff
    assert ko.pair_distances(a, b)[0, 0] == acc
