"""CPU oracle for the PCA initialisation of the projection -- TEST INFRASTRUCTURE, NOT PRODUCT.

Section 3.5 of the paper (arxiv 2505.15511) starts the optimisation from a PCA of the data.  This file writes that
out: the scores of the points on the first two principal axes.

Readings where the paper is silent:
  * the axes are the eigenvectors of the covariance C = (1/n) sum_i (x_i - mean)(x_i - mean)^T with the two largest
    eigenvalues lambda_1 >= lambda_2, everything in float64 from the float32 data;
  * an eigenvector's sign is free: each axis is oriented so that its entry of largest magnitude (the first one among
    equals) is positive;
  * the scale is the caller's: with std0 > 0 both coordinates are multiplied by std0 / sqrt(lambda_1), so that the first
    coordinate has standard deviation std0 (the usual small start of neighbour-embedding methods); std0 <= 0 leaves the
    scores as they are;
  * the result is rounded to float32 once, at the end.

parity status: pinned in tests/test_oracle_pca.py (scikit-learn's PCA, the singular value decomposition route,
planted axes, a cross-shaped example by hand, invariances)."""
from __future__ import annotations

import numpy as np


def orient(v: np.ndarray) -> np.ndarray:
    """The vector or its negative: whichever makes the first entry of largest magnitude positive."""
    return v if v[int(np.argmax(np.abs(v)))] > 0 else -v


def principal_axes(X: np.ndarray, n_components: int = 2):
    """(mean [d], eigenvalues [n_components] descending, axes [d, n_components] oriented), float64."""
    X64 = np.asarray(X, dtype=np.float32).astype(np.float64)
    n = len(X64)
    mean = X64.sum(axis=0) / n
    Xc = X64 - mean
    C = (Xc.T @ Xc) / n
    w, V = np.linalg.eigh(C)                      # ascending
    order = np.argsort(-w, kind="stable")[:n_components]
    axes = np.stack([orient(V[:, c]) for c in order], axis=1)
    return mean, w[order], axes


def pca_init(X: np.ndarray, std0: float = 0.0):
    """(theta0 float32 [n, 2], eigenvalues float64 [2])."""
    mean, lam, axes = principal_axes(X, 2)
    scores = (np.asarray(X, dtype=np.float32).astype(np.float64) - mean) @ axes
    if std0 > 0:
        scores = scores * (float(std0) / np.sqrt(lam[0]))
    return scores.astype(np.float32), lam
