"""Neighbourhood preservation@k between a reference neighbour list and the exact kNN of a 2-D
embedding (harness metric, computed with torch on whatever device is available)."""
import numpy as np
import torch


def knn_2d(theta, queries, k, device=None, block=1024):
    """Exact k nearest neighbours (self excluded) in the embedding for the listed query points."""
    device = device or ("cuda" if torch.cuda.is_available() else "cpu")
    th = torch.as_tensor(np.asarray(theta), dtype=torch.float64, device=device)
    q = torch.as_tensor(np.asarray(queries), dtype=torch.int64, device=device)
    out = torch.empty(len(q), k, dtype=torch.int64, device=device)
    for b0 in range(0, len(q), block):
        idx = q[b0:b0 + block]
        d = ((th[idx, None, :] - th[None, :, :]) ** 2).sum(-1)
        d[torch.arange(len(idx), device=device), idx] = float("inf")
        out[b0:b0 + block] = torch.topk(d, k, dim=1, largest=False).indices
    return out.cpu().numpy()


def neighbourhood_preservation(theta, ref_nbrs, k, queries=None):
    """(1/|Q|) sum_{i in Q} |N_k^ref(i) & N_k^2D(i)| / k."""
    n = len(theta)
    queries = np.arange(n) if queries is None else np.asarray(queries)
    low = knn_2d(theta, queries, k)
    ref = np.asarray(ref_nbrs)[queries][:, :k]
    hits = 0
    for a, b in zip(ref, low):
        hits += len(set(a.tolist()) & set(b.tolist()))
    return hits / (k * len(queries))
