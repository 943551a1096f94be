"""CPU oracle for the two quality measures of Section 4 -- TEST INFRASTRUCTURE, NOT PRODUCT.

Section 4 of the paper (arxiv 2505.15511) scores a projection by
  * neighbourhood preservation at k: the average overlap between the k-neighbourhoods of a point in the two spaces;
  * random triplet accuracy: the probability that a random triplet of points has the same ordering of its pairwise
    distances in the two spaces.
This file writes both out for float32 data X [n, d] (the high-dimensional space) and Y [n, d_low] (the projection).

Readings where the paper is silent:
  * distance of two float32 rows: the sum over the dimensions t = 0..d-1, in that order, of (x_t - y_t)^2 with every
    operation in float64 (the definition the nearest-neighbour oracle uses);
  * neighbourhoods: exact, the point itself excluded, ties to the lower point index; evaluated on the query points
    the caller lists (all points, or a seeded sample at large n); the result is the number of common neighbours
    summed over the queries ("hits"), the measure itself is hits / (k * queries);
  * a triplet is an anchor i and two other points j, k, all three distinct and uniform: triplet number t takes the
    words (o0, o1, o2, .) = Philox4x32-10(counter = (lo32(t), hi32(t), 0x54524950, 0), key = (lo32(seed), hi32(seed)))
    and i = floor(o0 n / 2^32); j = floor(o1 (n-1) / 2^32), moved up by one if >= i; k = floor(o2 (n-2) / 2^32), moved
    up by one if >= min(i, j) and then by one more if >= max(i, j);
  * the triplet agrees when [D_X(i,j) < D_X(i,k)] and [D_Y(i,j) < D_Y(i,k)] are the same truth value; the accuracy is
    the agreeing fraction of the triplets drawn.

parity status: pinned in tests/test_oracle_metrics.py (scipy's k-d tree and distance matrices, enumeration of all
triplets on tiny inputs, closed forms)."""
from __future__ import annotations

import numpy as np

from .knn_oracle import pair_distances
from .nomad_oracle import philox4x32_10_array

TRIPLET_STREAM = 0x54524950


def random_triplets(n: int, n_triplets: int, seed: int, first: int = 0):
    """(i, j, k) int64 arrays for triplets first .. first + n_triplets - 1: distinct, each ordered triple equally likely."""
    if n < 3:
        raise ValueError("a triplet needs three distinct points")
    t = np.arange(first, first + n_triplets, dtype=np.uint64)
    o0, o1, o2, _ = philox4x32_10_array(t & np.uint64(0xFFFFFFFF), t >> np.uint64(32), TRIPLET_STREAM, 0,
                                        seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    s32 = np.uint64(32)
    i = ((o0 * np.uint64(n)) >> s32).astype(np.int64)
    j = ((o1 * np.uint64(n - 1)) >> s32).astype(np.int64)
    j = j + (j >= i)
    k = ((o2 * np.uint64(n - 2)) >> s32).astype(np.int64)
    lo, hi = np.minimum(i, j), np.maximum(i, j)
    k = k + (k >= lo)
    k = k + (k >= hi)
    return i, j, k


def row_distances(A: np.ndarray, a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Squared distances between rows a[m] and b[m] of A, accumulated dimension by dimension in float64."""
    A = np.asarray(A, dtype=np.float32)
    acc = np.zeros(len(a), dtype=np.float64)
    for t in range(A.shape[1]):
        col = A[:, t].astype(np.float64)
        diff = col[a] - col[b]
        acc = acc + diff * diff
    return acc


def random_triplet_accuracy(X: np.ndarray, Y: np.ndarray, n_triplets: int, seed: int, chunk: int = 1 << 20):
    """(agreeing triplets, accuracy)."""
    n = len(X)
    agree = 0
    for first in range(0, n_triplets, chunk):
        m = min(chunk, n_triplets - first)
        i, j, k = random_triplets(n, m, seed, first)
        high = row_distances(X, i, j) < row_distances(X, i, k)
        low = row_distances(Y, i, j) < row_distances(Y, i, k)
        agree += int(np.count_nonzero(high == low))
    return agree, agree / n_triplets


def exact_neighbours(A: np.ndarray, queries: np.ndarray, k: int, block: int = 256) -> np.ndarray:
    """The k nearest other points of every query (ascending (distance, index)); -1 where fewer than k exist."""
    A = np.asarray(A, dtype=np.float32)
    n = len(A)
    out = np.full((len(queries), k), -1, dtype=np.int64)
    for b0 in range(0, len(queries), block):
        q = np.asarray(queries[b0:b0 + block], dtype=np.int64)
        D = pair_distances(A[q], A)
        D[np.arange(len(q)), q] = np.inf                       # a point is not its own neighbour
        order = np.lexsort((np.broadcast_to(np.arange(n), D.shape), D), axis=1)[:, :k]
        found = np.take_along_axis(D, order, axis=1) < np.inf
        out[b0:b0 + len(q), :order.shape[1]] = np.where(found, order, -1)
    return out


def neighbourhood_preservation(X: np.ndarray, Y: np.ndarray, k: int, queries=None):
    """(hits, hits / (k * queries)): common members of the two k-neighbourhoods, summed over the queries."""
    queries = np.arange(len(X)) if queries is None else np.asarray(queries, dtype=np.int64)
    high = exact_neighbours(X, queries, k)
    low = exact_neighbours(Y, queries, k)
    hits = 0
    for a, b in zip(high, low):
        hits += len((set(a.tolist()) & set(b.tolist())) - {-1})
    return hits, hits / (k * len(queries))
