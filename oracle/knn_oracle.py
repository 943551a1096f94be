"""CPU oracle for the in-cluster exact nearest-neighbour index -- TEST INFRASTRUCTURE, NOT PRODUCT.

Section 3.2 of the paper (arxiv 2505.15511) builds its kNN graph from a K-Means partition: the candidates for a
point's neighbours are the points of its own cluster, and among those the nearest neighbours are exact.  This file
is that definition written out: for every point the k nearest other points of its cluster under the squared
Euclidean distance.

Readings where the paper is silent:
  * distance of two fp32 rows: sum over the dimensions t = 0, 1, ..., d-1, in that order, of (x_t - y_t)^2 with every
    operation in float64 (difference, product, running sum each rounded once);
  * ties in distance go to the lower point index; a point is not its own neighbour; duplicates are ordinary points;
  * a cluster with fewer than k+1 points yields fewer than k neighbours: the remaining slots hold -1.

parity status: pinned in tests/test_oracle_knn.py (scipy's k-d tree per cluster, hand-made examples, ties)."""
from __future__ import annotations

import numpy as np


def pair_distances(Xq: np.ndarray, Xc: np.ndarray) -> np.ndarray:
    """Squared Euclidean distances [len(Xq), len(Xc)] accumulated dimension by dimension in float64."""
    q = np.asarray(Xq, dtype=np.float32).astype(np.float64)
    c = np.asarray(Xc, dtype=np.float32).astype(np.float64)
    acc = np.zeros((len(q), len(c)), dtype=np.float64)
    for t in range(q.shape[1]):
        diff = q[:, t][:, None] - c[:, t][None, :]
        acc = acc + diff * diff
    return acc


def in_cluster_knn(X: np.ndarray, cluster_of: np.ndarray, k: int, block: int = 512):
    """nbrs int64 [n, k] (ascending distance, ties by index, -1 where the cluster is too small) and dist float64 [n, k]
    (inf in the empty slots)."""
    X = np.asarray(X, dtype=np.float32)
    cluster_of = np.asarray(cluster_of, dtype=np.int64)
    n = len(X)
    nbrs = np.full((n, k), -1, dtype=np.int64)
    dist = np.full((n, k), np.inf, dtype=np.float64)
    for r in np.unique(cluster_of):
        members = np.nonzero(cluster_of == r)[0]          # ascending point index
        for b0 in range(0, len(members), block):
            q = members[b0:b0 + block]
            D = pair_distances(X[q], X[members])
            D[np.arange(len(q)), b0 + np.arange(len(q))] = np.inf          # not its own neighbour
            order = np.argsort(D, axis=1, kind="stable")                    # stable: ties keep the lower index first
            take = min(k, len(members) - 1)
            for row, i in enumerate(q):
                sel = order[row, :take]
                nbrs[i, :take] = members[sel]
                dist[i, :take] = D[row, sel]
    return nbrs, dist
