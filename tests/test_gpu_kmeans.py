"""nomad_kmeans_lloyd against the oracle: labels bit for bit, centroids bit for bit (the M step adds in the oracle's
order), iteration by iteration from the same centroids and as a whole run."""
import numpy as np
import pytest
import torch

from oracle import kmeans_oracle as km
from paper_2505_15511_amd import NomadError, kmeans_lloyd, workloads

pytestmark = pytest.mark.gpu


def note(msg):
    print(msg, flush=True)


def _data(n, d, comps, seed):
    X, _ = workloads.gmm_points(n, d, comps, 16.0, seed, mix="dirichlet", interleave=True)
    return X.numpy()


@pytest.mark.parametrize("n,d,K", [(5000, 16, 7), (8000, 64, 40), (3000, 130, 300), (2000, 5, 1), (4000, 768, 12)])
def test_one_iteration_matches_the_oracle_exactly(n, d, K):
    note(f"kmeans one step n={n} d={d} K={K}")
    X = _data(n, d, max(2, K // 3), 200 + d)
    rng = np.random.default_rng(K)
    C0 = X[rng.choice(n, K, replace=False)].copy()
    lab_ref, dist_ref = km.assign(X, C0)
    C_ref = km.update(X, lab_ref, C0)
    C, lab, it, inertia = kmeans_lloyd(X, C0, 1)
    assert it == 1 and np.array_equal(lab.astype(np.int64), lab_ref)
    assert np.array_equal(C, C_ref)
    assert abs(inertia - dist_ref.sum()) < 1e-9 * dist_ref.sum()


def test_full_run_matches_the_oracle_and_converges():
    n, d, K = 6000, 24, 12
    X = _data(n, d, 12, 300)
    C0 = X[np.random.default_rng(1).choice(n, K, replace=False)].copy()
    C_ref, lab_ref, it_ref, inertia_ref = km.lloyd(X, C0, 100)
    C, lab, it, inertia = kmeans_lloyd(torch.from_numpy(X).cuda(), torch.from_numpy(C0).cuda(), 100)
    note(f"  converged after {it} E steps (oracle {it_ref}), inertia {inertia:.6e}")
    assert it == it_ref and it < 100
    assert np.array_equal(lab.cpu().numpy().astype(np.int64), lab_ref) and np.array_equal(C.cpu().numpy(), C_ref)
    assert abs(inertia - inertia_ref) < 1e-9 * inertia_ref
    # stopping early gives the oracle's intermediate state
    C3_ref, lab3_ref, it3, _ = km.lloyd(X, C0, 3)
    C3, lab3, it3g, _ = kmeans_lloyd(X, C0, 3)
    assert it3 == it3g == 3 and np.array_equal(lab3.astype(np.int64), lab3_ref) and np.array_equal(C3, C3_ref)


def test_duplicate_centroids_empty_clusters_and_ties():
    rng = np.random.default_rng(7)
    X = rng.integers(0, 4, size=(1500, 3)).astype(np.float32)            # grid points: exact ties in bulk
    C0 = np.array([[0, 0, 0], [3, 3, 3], [0, 0, 0], [1.5, 1.5, 1.5], [50, 50, 50]], dtype=np.float32)   # a duplicate, a far one
    C_ref, lab_ref, it_ref, _ = km.lloyd(X, C0, 20)
    C, lab, it, _ = kmeans_lloyd(X, C0, 20)
    assert it == it_ref and np.array_equal(lab.astype(np.int64), lab_ref) and np.array_equal(C, C_ref)
    assert not (lab == 4).any() and np.array_equal(C[4], C0[4])           # the far centroid stays empty and where it was
    C1, lab1, _, _ = kmeans_lloyd(X, C0, 1)
    assert not (lab1 == 2).any() and np.array_equal(C1[2], C0[2])         # in the first E step the duplicate loses every tie


def test_bad_arguments_are_codes():
    X = np.zeros((10, 4), np.float32)
    with pytest.raises(NomadError):
        kmeans_lloyd(X, np.zeros((11, 4), np.float32), 5)        # more centroids than points
    with pytest.raises(NomadError):
        kmeans_lloyd(X, np.zeros((2, 4), np.float32), 0)


# ---------------------------------------------------------------- the start from a locality-sensitive hash
@pytest.mark.parametrize("n,d,K,b", [(5000, 16, 8, 3), (8000, 64, 40, 6), (3000, 130, 300, 9), (2000, 5, 1, 1), (4000, 768, 12, 4), (300, 7, 300, 30)])
def test_hash_start_matches_the_oracle_exactly(n, d, K, b):
    from paper_2505_15511_amd import kmeans_lsh_init
    note(f"kmeans hash start n={n} d={d} K={K} planes={b}")
    X = _data(n, d, 5, 400 + d)
    rng = np.random.default_rng(K)
    planes = rng.normal(size=(b, d)).astype(np.float32)
    anchors = rng.choice(n, b, replace=b > n).astype(np.int32)
    C_ref, buckets_ref = km.lsh_init(X, planes, anchors, K)
    C, buckets = kmeans_lsh_init(X, K, planes, anchors, return_buckets=True)
    assert np.array_equal(buckets.astype(np.int64), buckets_ref)
    assert np.array_equal(C, C_ref)
    Cd, bd = kmeans_lsh_init(torch.from_numpy(X).cuda(), K, torch.from_numpy(planes).cuda(), torch.from_numpy(anchors).cuda(), return_buckets=True)
    assert np.array_equal(Cd.cpu().numpy(), C_ref) and np.array_equal(bd.cpu().numpy().astype(np.int64), buckets_ref)


def test_hash_start_on_a_grid_and_bad_arguments():
    from paper_2505_15511_amd import kmeans_lsh_init
    # integer grid with integer normals: many points lie exactly on a plane (sum = 0 -> bit 0) and several buckets are empty
    rng = np.random.default_rng(6)
    G = rng.integers(0, 3, size=(2000, 4)).astype(np.float32)
    planes = rng.integers(-1, 2, size=(5, 4)).astype(np.float32)
    anchors = rng.choice(2000, 5).astype(np.int32)
    C_ref, b_ref = km.lsh_init(G, planes, anchors, 32)
    C, b = kmeans_lsh_init(G, 32, planes, anchors, return_buckets=True)
    assert np.array_equal(b.astype(np.int64), b_ref) and np.array_equal(C, C_ref)
    assert len(np.unique(b_ref)) < 32                                             # the empty-bucket rule was exercised
    with pytest.raises(NomadError):
        kmeans_lsh_init(G, 64, planes, anchors)                                   # 2^5 < 64
    with pytest.raises(NomadError):
        kmeans_lsh_init(G, 8, planes, np.array([0, 1, 2, 3, 2000], dtype=np.int32))   # an anchor that is no data point
    # the hash start feeds Lloyd's iterations, which agree with the oracle from it
    X = _data(6000, 24, 12, 301)
    pl = np.random.default_rng(1).normal(size=(4, 24)).astype(np.float32)
    an = np.array([5, 50, 500, 5000], dtype=np.int32)
    C0 = kmeans_lsh_init(X, 12, pl, an)
    C_ref, lab_ref, it_ref, _ = km.lloyd(X, km.lsh_init(X, pl, an, 12)[0], 30)
    Cg, lab, it, _ = kmeans_lloyd(X, C0, 30)
    assert it == it_ref and np.array_equal(lab.astype(np.int64), lab_ref) and np.array_equal(Cg, C_ref)


@pytest.mark.parametrize("n,d,K,b", [(5000, 16, 8, 3), (8000, 64, 40, 6), (700, 130, 300, 9), (4000, 768, 12, 4), (3, 5, 2, 1)])
def test_hash_start_with_median_anchors_matches_the_oracle_exactly(n, d, K, b):
    from paper_2505_15511_amd import kmeans_lsh_init
    note(f"kmeans hash start, median anchors n={n} d={d} K={K} planes={b}")
    X = _data(n, d, 5, 500 + d)
    planes = np.random.default_rng(K + 1).normal(size=(b, d)).astype(np.float32)
    anchors = km.lsh_median_anchors(X, planes)
    C_ref, buckets_ref = km.lsh_init(X, planes, anchors, K)
    C, buckets = kmeans_lsh_init(X, K, planes, None, return_buckets=True)
    assert np.array_equal(buckets.astype(np.int64), buckets_ref) and np.array_equal(C, C_ref)
    Cd, bd = kmeans_lsh_init(torch.from_numpy(X).cuda(), K, torch.from_numpy(planes).cuda(), None, return_buckets=True)
    assert np.array_equal(Cd.cpu().numpy(), C_ref) and np.array_equal(bd.cpu().numpy().astype(np.int64), buckets_ref)
    # ties in the projections (an integer grid): the rank rule decides alike on both sides
    G = np.random.default_rng(n).integers(0, 3, size=(min(n, 2000), 4)).astype(np.float32)
    pl = np.random.default_rng(b).integers(-1, 2, size=(3, 4)).astype(np.float32)
    Cg_ref, bg_ref = km.lsh_init(G, pl, km.lsh_median_anchors(G, pl), min(8, len(G)))
    Cg, bg = kmeans_lsh_init(G, min(8, len(G)), pl, None, return_buckets=True)
    assert np.array_equal(bg.astype(np.int64), bg_ref) and np.array_equal(Cg, Cg_ref)


def order_sensitive_points(n, d, K, seed):
    """Points whose cluster is fixed by column 0 (centroid j sits at 4096 j, the other columns of every centroid are 0), with
    columns 1.. built so that a cluster's float64 sum depends on the order of its additions: in every cluster and column an
    even number of members carry +-2^30 in cancelling pairs and the rest values near 2^-30, which a running sum that stands
    at a multiple of 2^30 absorbs and one that stands at zero keeps."""
    rng = np.random.default_rng(seed)
    member_of = rng.integers(0, K, n)
    X = np.zeros((n, d), dtype=np.float32)
    X[:, 0] = 4096.0 * member_of
    X[:, 1:] = (rng.uniform(-1, 1, (n, d - 1)) * 2.0 ** -30).astype(np.float32)
    for j in range(K):
        idx = np.flatnonzero(member_of == j)
        for col in range(1, d):
            q = len(idx) // 4
            pick = rng.choice(idx, 2 * q, replace=False)
            X[pick[:q], col] = 2.0 ** 30
            X[pick[q:], col] = -(2.0 ** 30)
    C0 = np.zeros((K, d), dtype=np.float32)
    C0[:, 0] = 4096.0 * np.arange(K)
    return X, C0, member_of


@pytest.mark.parametrize("n,d,K", [(20000, 6, 40), (20000, 4, 300), (60000, 3, 3000)])
def test_m_step_adds_in_ascending_point_order(n, d, K):
    """Centroids equal to the oracle's bit for bit on rows whose sums depend on the order of the additions: the points of
    every cluster were added in ascending point order (one radix pass of the sort for K <= 256, two beyond)."""
    note(f"kmeans M-step order n={n} d={d} K={K}")
    X, C0, member_of = order_sensitive_points(n, d, K, K)
    lab_ref, _ = km.assign(X, C0)
    assert np.array_equal(lab_ref, member_of)
    C_ref = km.update(X, lab_ref, C0)
    # the test has teeth: the same rows added in descending order give other numbers in most clusters
    C_rev = km.update(X[::-1], lab_ref[::-1], C0)
    assert (C_rev[:, 1:] != C_ref[:, 1:]).mean() > 0.5
    C, lab, it, _ = kmeans_lloyd(X, C0, 1)
    assert it == 1 and np.array_equal(lab.astype(np.int64), lab_ref)
    assert np.array_equal(C, C_ref)


def test_more_clusters_than_two_radix_digits():
    """Labels beyond 65,535: three radix passes of the M step's sort.  The nearest centroid of every point is known by
    construction (distance 0 in column 0 against at least 4096^2), so the E step of the oracle is not needed at this size."""
    n, d, K = 140000, 2, 66000
    X, C0, member_of = order_sensitive_points(n, d, K, 9)
    C_ref = km.update(X, member_of, C0)
    C, lab, it, _ = kmeans_lloyd(X, C0, 1)
    assert it == 1 and member_of.max() > 65535 and np.array_equal(lab.astype(np.int64), member_of)
    assert np.array_equal(C, C_ref)
