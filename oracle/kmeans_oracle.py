"""CPU oracle for the Lloyd iterations of the K-Means index -- TEST INFRASTRUCTURE, NOT PRODUCT.

Section 3.2 of the paper (arxiv 2505.15511): the index is a K-Means clustering, "expectation maximization until
convergence" from an initialisation that the caller supplies here (the paper's locality-sensitive-hash start is not
specified further).  One iteration, written out:

  E step   a_i = argmin_j D(x_i, c_j), D the squared Euclidean distance accumulated over t = 0..d-1 in order with
           every operation in float64 (the definition of oracle/knn_oracle.py); ties go to the lower j;
  M step   c_j = float32( (sum of the rows of cluster j, in float64, in ascending point order) / n_j ); a cluster
           that received no point keeps its centroid.

Iterations stop when an E step changes no assignment (the centroids are then a fixed point) or after max_iters.

The start from a locality-sensitive hash (one sentence in the paper, no detail) is read as random-hyperplane hashing:
  * b hyperplanes, 2^b >= K; plane j has the normal h_j (float32, drawn by the caller) and passes through the data
    point x_{a_j} (anchor indices drawn by the caller); bit j of a point is [ sum_t h_{j,t} (x_t - x_{a_j,t}) > 0 ], the
    sum over t = 0..d-1 in order, difference, product and running sum each rounded once in float64;
  * code = sum_j bit_j 2^j; bucket = floor(code K / 2^b); centroid j = the M step applied to bucket j;
  * an empty bucket j takes the data point with index floor(j n / K) as its centroid;
  * when the caller draws no anchors, plane j passes through the median of a sample along its normal: the sample is the
    m = min(1024, n) points floor(s n / m), their projections sum_t h_{j,t} x_t are accumulated over t = 0..d-1 in order
    (product and running sum each rounded once in float64), and the anchor is the sample point of rank floor(m / 2) in
    ascending (projection, point index): about half of the data on either side of every plane.

parity status: pinned in tests/test_oracle_kmeans.py (scipy's vq for the E step, closed forms, monotone inertia,
the fixed-point property; for the hash start: numpy's matrix product for the bits, planes with sides known by
construction, bucket means by a second route)."""
from __future__ import annotations

import numpy as np

from oracle.knn_oracle import pair_distances


def assign(X: np.ndarray, C: np.ndarray, block: int = 4096):
    """E step: (labels int64 [n], squared distance to the chosen centroid float64 [n])."""
    X = np.asarray(X, dtype=np.float32)
    C = np.asarray(C, dtype=np.float32)
    labels = np.zeros(len(X), dtype=np.int64)
    dist = np.zeros(len(X), dtype=np.float64)
    for b0 in range(0, len(X), block):
        D = pair_distances(X[b0:b0 + block], C)
        lab = np.argmin(D, axis=1)                      # first minimum: ties to the lower centroid
        labels[b0:b0 + block] = lab
        dist[b0:b0 + block] = D[np.arange(len(lab)), lab]
    return labels, dist


def update(X: np.ndarray, labels: np.ndarray, C_old: np.ndarray) -> np.ndarray:
    """M step: float32 means, rows added in ascending point order in float64; empty clusters keep their centroid."""
    X = np.asarray(X, dtype=np.float32)
    C = np.asarray(C_old, dtype=np.float32).copy()
    K = len(C)
    sums = np.zeros((K, X.shape[1]), dtype=np.float64)
    counts = np.zeros(K, dtype=np.int64)
    for i in range(len(X)):                             # ascending point order
        sums[labels[i]] = sums[labels[i]] + X[i].astype(np.float64)
        counts[labels[i]] += 1
    nz = counts > 0
    C[nz] = (sums[nz] / counts[nz, None].astype(np.float64)).astype(np.float32)
    return C


def lloyd(X: np.ndarray, C0: np.ndarray, max_iters: int):
    """Returns (centroids float32 [K,d], labels int64 [n], iterations run, inertia of the final labels against
    the centroids they were computed from)."""
    C = np.asarray(C0, dtype=np.float32).copy()
    labels = None
    it = 0
    inertia = float("nan")
    while it < max_iters:
        new_labels, dist = assign(X, C)
        it += 1
        inertia = float(dist.sum())
        if labels is not None and np.array_equal(new_labels, labels):
            break                                       # nothing moved: C is already the mean of these labels
        labels = new_labels
        C = update(X, labels, C)
    return C, labels, it, inertia


def lsh_buckets(X: np.ndarray, planes: np.ndarray, anchors: np.ndarray, K: int) -> np.ndarray:
    """Bucket int64 [n] of every point under the random-hyperplane hash (planes float32 [b, d], anchors int [b])."""
    X = np.asarray(X, dtype=np.float32)
    planes = np.asarray(planes, dtype=np.float32)
    b = len(planes)
    if (1 << b) < K:
        raise ValueError("2^planes must be at least K")
    code = np.zeros(len(X), dtype=np.int64)
    for j in range(b):
        a = X[int(anchors[j])].astype(np.float64)
        acc = np.zeros(len(X), dtype=np.float64)
        for t in range(X.shape[1]):
            diff = X[:, t].astype(np.float64) - a[t]
            acc = acc + np.float64(planes[j, t]) * diff
        code += (acc > 0).astype(np.int64) << j
    return (code * K) >> b


def lsh_init(X: np.ndarray, planes: np.ndarray, anchors: np.ndarray, K: int):
    """(centroids float32 [K, d], buckets int64 [n])."""
    X = np.asarray(X, dtype=np.float32)
    n = len(X)
    buckets = lsh_buckets(X, planes, anchors, K)
    fallback = X[(np.arange(K, dtype=np.int64) * n) // K]
    return update(X, buckets, fallback), buckets


LSH_SAMPLE = 1024


def lsh_median_anchors(X: np.ndarray, planes: np.ndarray) -> np.ndarray:
    """Anchor point int64 [b] of every plane: the median of a strided sample along the plane's normal."""
    X = np.asarray(X, dtype=np.float32)
    planes = np.asarray(planes, dtype=np.float32)
    n = len(X)
    m = min(LSH_SAMPLE, n)
    idx = (np.arange(m, dtype=np.int64) * n) // m
    anchors = np.zeros(len(planes), dtype=np.int64)
    for j in range(len(planes)):
        proj = np.zeros(m, dtype=np.float64)
        for t in range(X.shape[1]):
            proj = proj + np.float64(planes[j, t]) * X[idx, t].astype(np.float64)
        order = np.lexsort((idx, proj))
        anchors[j] = idx[order[m // 2]]
    return anchors
