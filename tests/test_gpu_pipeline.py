"""The composed method (K-Means -> in-cluster kNN -> graph -> PCA start -> epochs -> quality measures) end to end on
the GPU: the stages fit together, the embedding is better than its start and far better than chance."""
import numpy as np
import pytest
import torch

from paper_2505_15511_amd import pipeline, workloads

pytestmark = pytest.mark.gpu


def note(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("graph", ["directed", "symmetric"])
def test_project_and_evaluate(graph):
    n, d, comps = 30000, 32, 12
    X, _ = workloads.gmm_points(n, d, comps, 16.0, 21, mix="dirichlet", interleave=True)
    X = X.cuda()
    theta, info = pipeline.project(X, n_clusters=24, k=15, n_epochs=150, seed=3, graph=graph, return_info=True)
    assert theta.shape == (n, 2) and torch.isfinite(theta).all()
    nb = info["neighbours"]
    lab = info["labels"].long()
    ok = nb >= 0
    assert (lab[nb.clamp(min=0).long()] == lab[:, None])[ok].all()               # every edge stays inside its cluster
    assert info["edges"] >= int(ok.sum())
    np_start, ta_start = pipeline.evaluate(X, info["theta0"], n_queries=3000, n_triplets=200000, seed=1)
    np_end, ta_end = pipeline.evaluate(X, theta, n_queries=3000, n_triplets=200000, seed=1)
    note(f"  {graph}: R={info['n_clusters']} kmeans {info['kmeans_iterations']} its, E={info['edges']}, "
         f"NP@15 {np_start:.4f} -> {np_end:.4f}, triplets {ta_start:.4f} -> {ta_end:.4f}, seconds {info['seconds']}")
    assert np_end > 10 * 15 / n and np_end > np_start                            # chance is k / n
    assert ta_end > 0.6                                                          # global structure from the PCA start survives


def test_random_start_and_sampler_options_pass_through():
    X, _ = workloads.gmm_points(8000, 16, 6, 16.0, 22, mix="equal", interleave=True)
    X = X.cuda()
    theta = pipeline.project(X, n_clusters=8, n_epochs=40, init="random", kmeans_start="sample", seed=5, pool_size=256, pool_block=1024)
    assert theta.shape == (8000, 2) and torch.isfinite(theta).all()
    again = pipeline.project(X, n_clusters=8, n_epochs=40, init="random", kmeans_start="sample", seed=5, pool_size=256, pool_block=1024)
    assert torch.equal(theta, again)                                             # deterministic end to end


def test_small_clusters_leave_ragged_rows():
    # 60 points in 20 clusters: most clusters have fewer than k + 1 members, rows are shorter than k
    X, _ = workloads.gmm_points(60, 8, 3, 16.0, 23, mix="equal", interleave=True)
    nbrs = torch.tensor([[1, 2, -1], [0, -1, -1], [-1, -1, -1], [0, 1, 2]], dtype=torch.int32).cuda()
    row_ptr, col, w = pipeline.neighbour_lists_to_csr(nbrs, "directed")
    assert row_ptr.tolist() == [0, 2, 3, 3, 6] and col.tolist() == [1, 2, 0, 0, 1, 2]
    assert w is None                      # rows stay in rank order; the library derives p(j|i) from the ranks (Eq. 7)
    row_ptr, col, w = pipeline.neighbour_lists_to_csr(nbrs[:3], "symmetric")
    assert w is None and row_ptr.tolist() == [0, 2, 3, 4] and col.tolist() == [1, 2, 0, 0]
    theta = pipeline.project(X.cuda(), n_clusters=20, k=5, n_epochs=20, seed=1)
    assert torch.isfinite(theta).all()


def test_swiss_roll_local_structure_is_gained_and_global_structure_kept():
    """A rolled-up sheet in 20 dimensions: PCA cannot unroll it (low neighbourhood preservation, good triplet accuracy);
    the optimisation from the PCA start gains the neighbourhoods and keeps most of the global order, while a random
    start gains neighbourhoods only (Section 3.5's reason for the PCA start)."""
    rng = np.random.default_rng(0)
    n = 30000
    t = 1.5 * np.pi * (1 + 2 * rng.uniform(size=n))
    F = np.stack([t * np.cos(t), 21 * rng.uniform(size=n), t * np.sin(t)], axis=1)
    Q, _ = np.linalg.qr(rng.normal(size=(20, 20)))
    X = (np.concatenate([F, np.zeros((n, 17))], axis=1) @ Q.T + 0.05 * rng.normal(size=(n, 20))).astype(np.float32)
    X = torch.from_numpy(X).cuda()
    theta, info = pipeline.project(X, n_clusters=16, k=15, n_epochs=200, seed=1, return_info=True)
    np_start, ta_start = pipeline.evaluate(X, info["theta0"], n_queries=3000, n_triplets=200000, seed=1)
    np_end, ta_end = pipeline.evaluate(X, theta, n_queries=3000, n_triplets=200000, seed=1)
    rnd = pipeline.project(X, n_clusters=16, k=15, n_epochs=200, seed=1, init="random")
    np_rnd, ta_rnd = pipeline.evaluate(X, rnd, n_queries=3000, n_triplets=200000, seed=1)
    note(f"  swiss roll: NP@15 {np_start:.3f} -> {np_end:.3f} (random start {np_rnd:.3f}), "
         f"triplets {ta_start:.3f} -> {ta_end:.3f} (random start {ta_rnd:.3f})")
    assert np_start < 0.25 and np_end > 0.45 and np_end > 3 * np_start
    assert ta_end > 0.7 and ta_end > ta_rnd + 0.15
    assert np_rnd > 0.2
