"""The whole method of the paper on one GPU, composed from the library's entry points: K-Means partition (Section
3.2) -> exact nearest neighbours inside clusters -> the kNN graph of Section 3.1 -> PCA start (Section 3.5) -> NOMAD
epochs -> the quality measures of Section 4.  Every step with arithmetic in it runs in libnomad; this module only
passes device tensors from one entry point to the next and lays the neighbour lists out as CSR."""
from __future__ import annotations

import time

import numpy as np
import torch

from . import workloads
from .binding import (SCATTER_DETERMINISTIC, Nomad, kmeans_lloyd, kmeans_lsh_init, knn_in_clusters, neighbourhood_preservation, pca_init,
                      random_triplet_accuracy)


def neighbour_lists_to_csr(nbrs: torch.Tensor, graph: str = "directed"):
    """CSR of the kNN graph from neighbour lists [n, k] in rank order (-1 = no such neighbour).
    "directed": the paper's digraph, row i = i's out-neighbours in rank order (the library derives p(j|i) from the
    ranks, Eq. 7, when asked to: inverse_rank_weights); "symmetric": union with the transposed edges, unit weights.
    Returns (row_ptr, col_idx, None)."""
    n, k = nbrs.shape
    valid = nbrs >= 0
    if graph == "symmetric":
        src = torch.arange(n, device=nbrs.device, dtype=torch.int64)[:, None].expand(n, k)[valid]
        dst = nbrs[valid].to(torch.int64)
        key = torch.unique(torch.cat([src * n + dst, dst * n + src]))
        rows = torch.div(key, n, rounding_mode="floor")
        counts = torch.bincount(rows, minlength=n)
        col, w = (key - rows * n).to(torch.int32), None
    elif graph == "directed":
        counts = valid.sum(dim=1)
        col = nbrs[valid].to(torch.int32).contiguous()
        w = None                                                   # rows stay in rank order: the library weighs them (Eq. 7)
    else:
        raise ValueError("graph must be 'directed' or 'symmetric'")
    row_ptr = torch.zeros(n + 1, dtype=torch.int64, device=nbrs.device)
    torch.cumsum(counts, 0, out=row_ptr[1:])
    if int(row_ptr[-1]) >= 2 ** 31:
        raise ValueError("edge count does not fit int32 offsets")
    return row_ptr.to(torch.int32), col, w


def project(X: torch.Tensor, n_clusters: int, k: int = 15, n_epochs: int = 200, n_neg: int = 5, noise_count: float = 0.0,
            lr0: float = 1.0, seed: int = 0, kmeans_iters: int = 25, init: str = "pca", std0: float = 0.01,
            graph: str = "directed", kmeans_start: str = "lsh", device: int = 0, return_info: bool = False, **nomad_options):
    """Project the rows of X (float32 tensor on the GPU) to the plane.  Returns theta [n, 2] on the device, and with
    return_info a dict of the intermediate results and the seconds each stage took.

    kmeans_start "lsh": the centroids start as the bucket means of a random-hyperplane hash (ceil(log2 n_clusters) planes
    with Gaussian normals drawn here with the seed, each through the median of a sample along its normal); "sample": as n_clusters of the
    points.  Clusters that end up empty are dropped.  Remaining keyword arguments go to Nomad (pool_size,
    sampled_far_field, batches_per_epoch, ...)."""
    if not (X.is_cuda and X.dtype == torch.float32 and X.dim() == 2):
        raise ValueError("X must be a float32 [n, d] tensor on the GPU")
    n = X.shape[0]
    times = {}

    def timed(name, fn):
        torch.cuda.synchronize(device)
        t0 = time.perf_counter()
        out = fn()
        torch.cuda.synchronize(device)
        times[name] = time.perf_counter() - t0
        return out

    gen = torch.Generator().manual_seed(seed)
    if kmeans_start == "lsh":
        b = max(1, int(np.ceil(np.log2(n_clusters))))
        planes = torch.randn(b, X.shape[1], generator=gen, dtype=torch.float32).to(X.device)
        start = timed("kmeans_start", lambda: kmeans_lsh_init(X, n_clusters, planes, None, device=device))   # planes through sample medians
    elif kmeans_start == "sample":
        start = X[torch.randperm(n, generator=gen)[:n_clusters].to(X.device)]
    else:
        raise ValueError("kmeans_start must be 'lsh' or 'sample'")
    _, labels, km_iters, inertia = timed("kmeans", lambda: kmeans_lloyd(X, start, kmeans_iters, device=device))
    used, labels = torch.unique(labels, return_inverse=True)
    labels = labels.to(torch.int32)
    R = int(used.numel())
    nbrs = timed("knn", lambda: knn_in_clusters(X, labels, R, k, device=device))
    row_ptr, col, w = timed("graph", lambda: neighbour_lists_to_csr(nbrs, graph))
    if init == "pca":
        theta0 = timed("init", lambda: pca_init(X, std0, device=device))
    elif init == "random":
        theta0 = workloads.init_embedding(n, seed, std0, device=X.device)
    else:
        raise ValueError("init must be 'pca' or 'random'")
    with Nomad(n, R, n_neg, noise_count, n_epochs, lr0, seed, SCATTER_DETERMINISTIC, device,
               inverse_rank_weights=(graph == "directed"), **nomad_options) as nm:
        timed("set_graph", lambda: (nm.set_graph(row_ptr, col, w, labels, None), nm.set_embedding(theta0)))

        def run():
            for t in range(n_epochs):
                nm.epoch(t)
        timed("epochs", run)
        theta = nm.get_embedding(device=True)
    if return_info:
        return theta, dict(labels=labels, n_clusters=R, kmeans_iterations=km_iters, inertia=inertia, neighbours=nbrs,
                           edges=int(col.numel()), theta0=theta0, seconds=times)
    return theta


def evaluate(X: torch.Tensor, theta: torch.Tensor, k: int = 15, n_queries: int = 10000, n_triplets: int = 1_000_000, seed: int = 0,
             device: int = 0):
    """(neighbourhood preservation at k on a seeded sample of queries, random triplet accuracy), Section 4."""
    n = X.shape[0]
    q = None
    if n_queries < n:
        q = torch.randperm(n, generator=torch.Generator().manual_seed(seed))[:n_queries].to(torch.int32).to(X.device)
    _, preservation = neighbourhood_preservation(X, theta, k, q, device=device)
    _, accuracy = random_triplet_accuracy(X, theta, n_triplets, seed, device=device)
    return preservation, accuracy
