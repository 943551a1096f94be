"""nomad_knn_in_clusters against the oracle's float64 definition: neighbour lists bit for bit."""
import numpy as np
import pytest
import torch

from oracle import knn_oracle as ko
from paper_2505_15511_amd import NomadError, knn_in_clusters, workloads

pytestmark = pytest.mark.gpu


def note(msg):
    print(msg, flush=True)


def _gmm(n, d, comps, seed, interleave=True):
    X, c = workloads.gmm_points(n, d, comps, 16.0, seed, mix="dirichlet", interleave=interleave)
    return X.numpy(), c.numpy()


@pytest.mark.parametrize("n,d,comps,k", [(3000, 50, 10, 15), (6000, 128, 7, 15), (2500, 7, 3, 32), (1500, 300, 4, 10), (900, 768, 2, 5),
                                         (4000, 33, 1, 1), (1301, 400, 5, 32), (1103, 700, 3, 20), (977, 330, 3, 15), (1999, 512, 2, 8),
                                         (1500, 260, 1, 15)])
def test_neighbours_match_the_oracle_bit_for_bit(n, d, comps, k):
    note(f"knn n={n} d={d} clusters={comps} k={k}")
    X, c = _gmm(n, d, comps, 100 + d)
    ref, _ = ko.in_cluster_knn(X, c, k)
    out, st = knn_in_clusters(torch.from_numpy(X).cuda(), torch.from_numpy(c).cuda(), comps, k, return_stats=True)
    note(f"  fallback queries {st['fallback_queries']} of {n}")
    assert np.array_equal(out.cpu().numpy().astype(np.int64), ref)
    assert st["fallback_queries"] < n // 100           # the matrix-core filter decides nearly everything
    host = knn_in_clusters(X, c, comps, k)              # host buffers in, host buffer out
    assert np.array_equal(host.astype(np.int64), ref)


def test_ragged_clusters_small_clusters_and_empty_ones():
    rng = np.random.default_rng(5)
    sizes = [1, 2, 3, 16, 17, 127, 128, 129, 300, 0, 1000]
    c = np.repeat(np.arange(len(sizes)), sizes)
    perm = rng.permutation(len(c))
    c = c[perm]
    X = rng.normal(size=(len(c), 20)).astype(np.float32)
    ref, _ = ko.in_cluster_knn(X, c, 15)
    out = knn_in_clusters(X, c, len(sizes), 15)
    assert np.array_equal(out.astype(np.int64), ref)
    assert (out[c == 0] == -1).all() and (out[c == 2][:, 2:] == -1).all()


def test_duplicates_and_exact_ties_take_the_exact_path():
    """Points on an integer grid, many of them repeated: distances tie exactly, in bulk; the answer is still the
    float64 definition with ties to the lower index."""
    rng = np.random.default_rng(6)
    X = rng.integers(0, 3, size=(1200, 4)).astype(np.float32)
    c = rng.integers(0, 2, 1200)
    ref, _ = ko.in_cluster_knn(X, c, 15)
    out, st = knn_in_clusters(X, c, 2, 15, return_stats=True)
    note(f"  fallback queries {st['fallback_queries']} of 1200")
    assert np.array_equal(out.astype(np.int64), ref)
    assert st["fallback_queries"] > 0


def test_far_from_the_origin_the_float32_filter_is_still_certified_or_replaced():
    """A large common offset makes the float32 keys coarse (|x|^2 ~ 1e8): whatever the filter cannot prove goes
    through the exact path."""
    X, c = _gmm(2000, 16, 4, 77)
    X = (X + 3000.0).astype(np.float32)
    ref, _ = ko.in_cluster_knn(X, c, 15)
    out, st = knn_in_clusters(X, c, 4, 15, return_stats=True)
    note(f"  fallback queries {st['fallback_queries']} of 2000")
    assert np.array_equal(out.astype(np.int64), ref)


def test_bad_arguments_are_codes():
    X = np.zeros((10, 4), np.float32)
    c = np.zeros(10, np.int32)
    for kw in (dict(k=0), dict(k=33), dict(n_clusters=0)):
        args = dict(n_clusters=1, k=3)
        args.update(kw)
        with pytest.raises(NomadError):
            knn_in_clusters(X, c, **args)
    with pytest.raises(NomadError):
        knn_in_clusters(np.zeros((10, 769), np.float32), c, 1, 3)
    with pytest.raises(NomadError):
        knn_in_clusters(X, np.full(10, 5, np.int32), 2, 3)       # cluster id out of range


def test_index_output_feeds_the_epoch_path():
    """Section 3.2 end to end on the device: clusters (given) -> in-cluster exact kNN -> symmetrised graph -> NOMAD
    epochs.  Every edge stays inside its cluster, and the embedding keeps the clusters' neighbourhoods."""
    from paper_2505_15511_amd import Nomad, SCATTER_DETERMINISTIC
    from tests.np_metric import neighbourhood_preservation
    n, d, comps, k = 20000, 64, 20, 15
    X, c = workloads.gmm_points(n, d, comps, 16.0, 9, mix="equal", interleave=True)
    nb = knn_in_clusters(X.cuda(), c.cuda(), comps, k)
    assert (nb >= 0).all()
    assert (c.cuda()[nb.long()] == c.cuda()[:, None]).all()                       # each cluster is a component of the graph
    row_ptr, col = workloads.knn_lists_to_symmetric_csr(n, nb.cpu())
    T = 100
    with Nomad(n, comps, 5, 5.0, T, 1.0, 1, SCATTER_DETERMINISTIC) as nm:
        nm.set_graph(row_ptr, col, None, c, None)
        nm.set_embedding(workloads.init_embedding(n, 3))
        L0 = nm.loss(0)
        for t in range(T):
            nm.epoch(t)
        L1 = nm.loss(T)
        theta = nm.get_embedding()
    q = np.random.default_rng(0).choice(n, 4000, replace=False)
    np15 = neighbourhood_preservation(theta, nb.cpu().numpy(), 15, q)
    note(f"  loss {L0:.4f} -> {L1:.4f}, NP@15 against the index's own neighbours {np15:.4f}")
    assert L1 < 0.5 * L0 and np15 > 0.02         # chance is 15 / 20000; isotropic blobs have little inner structure
