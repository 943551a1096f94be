"""The synthetic input generators produce what the workload recipe says."""
import numpy as np
import torch

from paper_2505_15511_amd import workloads as wl


def _check_csr(n, row_ptr, col):
    row_ptr, col = row_ptr.numpy().astype(np.int64), col.numpy().astype(np.int64)
    assert row_ptr[0] == 0 and row_ptr[-1] == len(col) and np.all(np.diff(row_ptr) >= 0)
    rows = np.repeat(np.arange(n), np.diff(row_ptr))
    assert np.all(rows != col) and col.min() >= 0 and col.max() < n
    key = rows * n + col
    assert np.all(np.diff(key) > 0)                       # sorted rows, no duplicates
    assert np.array_equal(np.sort(col * n + rows), key)   # symmetric
    return rows


def test_zipf_sizes():
    s = wl.zipf_cluster_sizes(1_000_000, 1024, 1.1, 17)
    assert s.sum() == 1_000_000 and s.min() >= 17 and np.all(np.diff(s) <= 0)
    assert 175_000 < s[0] < 183_000
    s = wl.zipf_cluster_sizes(2000, 50, 1.1, 17)
    assert s.sum() == 2000 and s.min() >= 17


def test_planted_graph_structure():
    n, R, k = 20000, 40, 15
    g = wl.planted_knn_graph(n, R, k, 0.02, seed=5)
    rows = _check_csr(n, g["row_ptr"], g["col_idx"])
    cl = g["cluster_of"].numpy()
    assert np.all(np.diff(cl) >= 0) and np.array_equal(np.bincount(cl, minlength=R), g["sizes"])
    out = g["out_nbrs"].numpy()
    assert out.shape == (n, k) and np.all(out != np.arange(n)[:, None])
    cross = (cl[out] != cl[:, None]).mean()
    assert 0.015 < cross < 0.025
    srt = np.sort(out, 1)
    assert (srt[:, 1:] == srt[:, :-1]).mean() < 1e-3      # distinct draws (cross edges may rarely collide)
    deg = np.diff(g["row_ptr"].numpy())
    assert deg.min() >= k - 1 and 1.9 * k < deg.mean() < 2.0 * k
    # same seed, same graph
    g2 = wl.planted_knn_graph(n, R, k, 0.02, seed=5)
    assert torch.equal(g["col_idx"], g2["col_idx"])


def test_config1_shape():
    w = wl.make_config(1)
    assert w.n == 2000 and w.n_clusters == 10 and w.n_neg == 5 and w.n_epochs == 100 and w.lr0 == 1.0
    _check_csr(w.n, w.row_ptr, w.col_idx)
    assert np.array_equal(np.bincount(w.cluster_of.numpy()), np.full(10, 200))
    assert w.theta0.dtype == torch.float32 and abs(float(w.theta0.std()) - 0.01) < 1e-3
    nb = w.out_nbrs.numpy().astype(np.int64)
    # exact kNN: check a few rows against a direct computation
    X = w.X.numpy().astype(np.float64)
    for i in (0, 17, 1999):
        d = ((X - X[i]) ** 2).sum(1)
        d[i] = np.inf
        assert set(np.argsort(d)[:15].tolist()) == set(nb[i].tolist())
    # neighbours overwhelmingly share the generating component
    assert (w.cluster_of.numpy()[nb] == w.cluster_of.numpy()[:, None]).mean() > 0.99


def test_scaled_config5_has_one_group_per_cluster():
    w = wl.make_config(5, scale=1e-3)
    assert w.n == 60000 and w.n_clusters == 16 and w.n_neg == 2 and w.noise_count == 5.0
    assert torch.equal(w.cluster_group, torch.arange(16, dtype=torch.int32))
    _check_csr(w.n, w.row_ptr, w.col_idx)


def test_balanced_groups():
    sizes = wl.zipf_cluster_sizes(100000, 64, 1.1, 17)
    g = wl.balanced_groups(sizes, 8)
    load = np.bincount(g, weights=sizes, minlength=8)
    assert load.max() <= max(sizes[0], 1.2 * load.mean())
