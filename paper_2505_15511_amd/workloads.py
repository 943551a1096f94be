"""Seeded synthetic workloads for the NOMAD Projection epoch path.

This module only *manufactures inputs* (point clouds, kNN graphs, cluster
labels, initial embeddings).  It holds none of the method's arithmetic: no
Cauchy kernel, no loss, no sampler.  Both the CPU oracle's tests and the HIP
library's tests feed from it so that they see identical arrays.

The paper's corpora (ArXiv, ImageNet, PubMed, Multilingual Wikipedia; Section 4)
are not available offline.  These generators stand in for them and keep the
structure the paper's ANN index produces (Section 3.2): a kNN graph whose edges
stay (almost entirely) inside K-Means-like clusters, a 2-D fp32 embedding, and
up to 60 M points.

All randomness comes from ``torch.Generator`` objects seeded explicitly; a
workload is a pure function of (config id, scale, device type).
"""
from __future__ import annotations

import dataclasses
from typing import Optional

import numpy as np
import torch


# --------------------------------------------------------------------------
# containers
# --------------------------------------------------------------------------
@dataclasses.dataclass
class Workload:
    """One problem instance.  Tensors live on ``device``; ``numpy()`` gives a
    host copy for the oracle."""

    name: str
    n: int
    row_ptr: torch.Tensor          # int32 [n+1]
    col_idx: torch.Tensor          # int32 [E], rows sorted ascending, no duplicates, no self loops
    cluster_of: torch.Tensor       # int32 [n]
    n_clusters: int
    theta0: torch.Tensor           # float32 [n,2]
    n_neg: int                     # s
    noise_count: float             # |M|
    n_epochs: int                  # T
    lr0: float
    seed: int                      # library / sampler seed
    cluster_group: Optional[torch.Tensor] = None   # int32 [n_clusters] or None
    weights: Optional[torch.Tensor] = None         # float32 [E] or None (unit)
    out_nbrs: Optional[torch.Tensor] = None        # int32 [n,k]: planted / exact kNN lists before symmetrisation
    X: Optional[torch.Tensor] = None               # float32 [n,dim] high-d points (GMM configs only)
    k: int = 15
    pool_size: int = 0             # opt-in pooled sampler: points per pool (0 = i.i.d. negatives per edge)
    pool_block: int = 0            # opt-in pooled sampler: consecutive CSR positions sharing a pool
    pool_mode: int = 0             # pooled sampler: 0 = 16-bit picks, 1 = distinct picks (exactly i.i.d. inside an edge)
    pool_line: int = 1             # distinct picks: consecutive points per pool line
    pool_segment: int = 64         # distinct picks: consecutive CSR positions dealt to a block together
    inverse_rank_weights: bool = False   # rows are in rank order and p(j|i) follows the inverse-rank model of Eq. 7
    batches_per_epoch: int = 1     # sequential sub-steps of an epoch over consecutive head ranges
    sampled_far_field: bool = False   # opt-in: the sum over approximated cells estimated from the samples
    mean_gradient: bool = False       # opt-in: the gradient also flows through the cell means

    @property
    def n_edges(self) -> int:
        return int(self.col_idx.numel())

    def numpy(self) -> dict:
        def h(t):
            return None if t is None else t.detach().cpu().numpy()
        return dict(
            n=self.n, row_ptr=h(self.row_ptr), col_idx=h(self.col_idx), weights=h(self.weights),
            cluster_of=h(self.cluster_of), n_clusters=self.n_clusters, cluster_group=h(self.cluster_group),
            theta0=h(self.theta0), n_neg=self.n_neg, noise_count=self.noise_count,
            n_epochs=self.n_epochs, lr0=self.lr0, seed=self.seed, pool_size=self.pool_size, pool_block=self.pool_block,
            pool_mode=self.pool_mode, pool_line=self.pool_line, pool_segment=self.pool_segment,
            inverse_rank_weights=self.inverse_rank_weights,
            batches_per_epoch=self.batches_per_epoch, sampled_far_field=self.sampled_far_field,
            mean_gradient=self.mean_gradient,
        )


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


# --------------------------------------------------------------------------
# Gaussian mixtures + exact kNN (configs 1-2)
# --------------------------------------------------------------------------
def gmm_points(n: int, dim: int, n_comp: int, mean_var: float, seed: int, *,
               mix: str = "equal", interleave: bool = True, device="cpu"):
    """Isotropic unit-variance Gaussian mixture.  Returns (X fp32 [n,dim], comp int32 [n]).

    ``mix='equal'`` gives n/n_comp points per component; ``'dirichlet'`` draws the mixture
    weights from Dirichlet(1).  With ``interleave`` the points are put in random order so the
    clusters are *not* contiguous in index space; otherwise they are numbered component by
    component."""
    g = _gen(seed, "cpu")
    means = torch.randn(n_comp, dim, generator=g, dtype=torch.float64) * float(np.sqrt(mean_var))
    if mix == "equal":
        comp = torch.arange(n, dtype=torch.int64) * n_comp // n
    elif mix == "dirichlet":
        e = -torch.log(torch.rand(n_comp, generator=g, dtype=torch.float64))
        w = e / e.sum()
        comp = torch.multinomial(w, n, replacement=True, generator=g)
        comp, _ = torch.sort(comp)
    else:
        raise ValueError(mix)
    if interleave:
        comp = comp[torch.randperm(n, generator=g)]
    X = means[comp] + torch.randn(n, dim, generator=g, dtype=torch.float64)
    return X.to(torch.float32).to(device), comp.to(torch.int32).to(device)


def exact_knn(X: torch.Tensor, k: int, block: int = 2048) -> torch.Tensor:
    """Exact Euclidean k nearest neighbours (self excluded, ties -> lower index) by blocked
    brute force.  Returns int32 [n,k] ordered by ascending distance."""
    n = X.shape[0]
    Xd = X.to(torch.float64) if X.device.type == "cpu" and n <= 20000 else X.to(torch.float32)
    sq = (Xd * Xd).sum(1)
    out = torch.empty(n, k, dtype=torch.int32, device=X.device)
    for b0 in range(0, n, block):
        b1 = min(n, b0 + block)
        d = sq[b0:b1, None] + sq[None, :] - 2.0 * (Xd[b0:b1] @ Xd.T)
        d[torch.arange(b1 - b0, device=X.device), torch.arange(b0, b1, device=X.device)] = float("inf")
        # stable sort on distance keeps the lower index first among ties
        _, idx = torch.topk(d, k, dim=1, largest=False, sorted=True)
        out[b0:b1] = idx.to(torch.int32)
    return out


def knn_lists_to_symmetric_csr(n: int, nbrs: torch.Tensor):
    """Union of a directed kNN list with its transpose, duplicates and self loops removed.
    Returns (row_ptr int32 [n+1], col_idx int32 [E]) with each row sorted ascending."""
    dev = nbrs.device
    k = nbrs.shape[1]
    src = torch.arange(n, device=dev, dtype=torch.int64).repeat_interleave(k)
    dst = nbrs.reshape(-1).to(torch.int64)
    keep = src != dst
    src, dst = src[keep], dst[keep]
    key = torch.cat([src * n + dst, dst * n + src])
    del src, dst, keep
    key = torch.unique(key)            # sorted ascending => rows in order, columns ascending
    rows = torch.div(key, n, rounding_mode="floor")
    cols = (key - rows * n).to(torch.int32)
    del key
    counts = torch.bincount(rows, minlength=n)
    del rows
    row_ptr = torch.zeros(n + 1, dtype=torch.int64, device=dev)
    torch.cumsum(counts, 0, out=row_ptr[1:])
    if int(row_ptr[-1]) >= 2 ** 31:
        raise ValueError("edge count does not fit int32 offsets")
    return row_ptr.to(torch.int32), cols


# --------------------------------------------------------------------------
# planted cluster graphs (configs 3-5)
# --------------------------------------------------------------------------
def zipf_cluster_sizes(n: int, n_clusters: int, exponent: float = 1.1, floor: int = 17) -> np.ndarray:
    """Cluster sizes proportional to rank**-exponent, rounded by largest remainder so that they
    sum to n, each at least ``floor`` (the deficit is taken from the largest cluster)."""
    if n < n_clusters * floor:
        raise ValueError("n too small for this many clusters")
    w = np.arange(1, n_clusters + 1, dtype=np.float64) ** (-exponent)
    ideal = n * w / w.sum()
    base = np.floor(ideal).astype(np.int64)
    rem = int(n - base.sum())
    order = np.argsort(-(ideal - base), kind="stable")
    base[order[:rem]] += 1
    short = np.maximum(0, floor - base)
    base = np.maximum(base, floor)
    base[0] -= int(short.sum())
    assert base.sum() == n and base.min() >= floor
    return base


def _k_distinct(pop: torch.Tensor, k: int, g: torch.Generator) -> torch.Tensor:
    """For every row draw a uniformly random k-subset of {0..pop-1} (Floyd's method, vectorised
    over rows).  pop: int64 [m] with pop >= k.  Returns int64 [m,k]."""
    m = pop.numel()
    dev = pop.device
    out = torch.empty(m, k, dtype=torch.int64, device=dev)
    for idx in range(k):
        j = pop - k + idx                                   # current top element
        t = torch.floor(torch.rand(m, generator=g, dtype=torch.float64, device=dev) * (j + 1).to(torch.float64)).to(torch.int64)
        t = torch.minimum(t, j)
        if idx:
            dup = (out[:, :idx] == t[:, None]).any(1)
            t = torch.where(dup, j, t)
        out[:, idx] = t
    return out


def planted_knn_graph(n: int, n_clusters: int, k: int, cross_frac: float, seed: int, device="cpu"):
    """Planted kNN graph: Zipf(1.1)-sized clusters numbered contiguously; every point draws k
    distinct out-neighbours uniformly from its own cluster (self excluded); each draw is
    independently, with probability ``cross_frac``, replaced by a uniform point of a uniformly
    chosen other cluster; the result is symmetrised and de-duplicated.

    Returns dict(row_ptr, col_idx, cluster_of, out_nbrs, sizes)."""
    sizes_np = zipf_cluster_sizes(n, n_clusters, 1.1, floor=k + 2)
    g = _gen(seed, device)
    sizes = torch.from_numpy(sizes_np).to(device)
    starts = torch.zeros(n_clusters + 1, dtype=torch.int64, device=device)
    torch.cumsum(sizes, 0, out=starts[1:])
    cluster_of = torch.repeat_interleave(torch.arange(n_clusters, device=device, dtype=torch.int64), sizes)
    my_start = starts[cluster_of]
    my_size = sizes[cluster_of]
    local = torch.arange(n, device=device, dtype=torch.int64) - my_start
    pick = _k_distinct(my_size - 1, k, g)                   # in [0, size-2]
    pick = pick + (pick >= local[:, None]).to(torch.int64)  # skip self
    nbrs = pick + my_start[:, None]
    del pick
    if cross_frac > 0 and n_clusters > 1:
        cross = torch.rand(n, k, generator=g, device=device) < cross_frac
        oc = torch.floor(torch.rand(n, k, generator=g, dtype=torch.float64, device=device) * (n_clusters - 1)).to(torch.int64)
        oc = torch.clamp(oc, max=n_clusters - 2)
        oc = oc + (oc >= cluster_of[:, None]).to(torch.int64)
        u = torch.rand(n, k, generator=g, dtype=torch.float64, device=device)
        op = starts[oc] + torch.minimum(torch.floor(u * sizes[oc].to(torch.float64)).to(torch.int64), sizes[oc] - 1)
        nbrs = torch.where(cross, op, nbrs)
        del cross, oc, u, op
    nbrs32 = nbrs.to(torch.int32)
    del nbrs
    row_ptr, col_idx = knn_lists_to_symmetric_csr(n, nbrs32)
    return dict(row_ptr=row_ptr, col_idx=col_idx, cluster_of=cluster_of.to(torch.int32),
                out_nbrs=nbrs32, sizes=sizes_np)


def directed_rank_csr(out_nbrs: torch.Tensor):
    """The kNN digraph as Section 3.1 has it: row i holds i's k out-neighbours in rank order (no transposed
    edges added).  Its edge probabilities follow from the ranks (Eq. 7): computing them is the library's part (and
    the oracle's), not the generator's.  Returns (row_ptr int32 [n+1], col_idx int32 [n k])."""
    n, k = out_nbrs.shape
    dev = out_nbrs.device
    row_ptr = (torch.arange(n + 1, dtype=torch.int64, device=dev) * k).to(torch.int32)
    return row_ptr, out_nbrs.reshape(-1).to(torch.int32).contiguous()


def init_embedding(n: int, seed: int, std: float = 0.01, device="cpu") -> torch.Tensor:
    """theta_0 ~ N(0, std^2 I) in fp32, generated on the host so that it does not depend on the device."""
    g = _gen(seed, "cpu")
    return (torch.randn(n, 2, generator=g, dtype=torch.float32) * std).to(device)


# --------------------------------------------------------------------------
# the five benchmark configurations
# --------------------------------------------------------------------------
_CONFIGS = {
    # id: (kind, n, dim/None, clusters, k, cross, s, |M|, T, grouped)
    1: dict(kind="gmm", n=2_000, dim=50, comps=10, mean_var=25.0, mix="equal", k=15, s=5, M=5.0, T=100),
    2: dict(kind="gmm", n=100_000, dim=128, comps=50, mean_var=16.0, mix="dirichlet", k=15, s=5, M=5.0, T=200),
    3: dict(kind="planted", n=1_000_000, clusters=1024, k=15, cross=0.02, s=5, M=5.0, T=200),
    4: dict(kind="planted", n=10_000_000, clusters=4096, k=15, cross=0.02, s=5, M=5.0, T=100),
    5: dict(kind="planted", n=60_000_000, clusters=16384, k=10, cross=0.01, s=2, M=5.0, T=50, own_group=True),
}


def make_config(cfg: int, *, scale: float = 1.0, device="cpu", n_groups: Optional[int] = None,
                paper_graph: bool = False) -> Workload:
    """Build benchmark configuration ``cfg`` (1-5).

    ``scale`` < 1 shrinks n (and, for the planted graphs, the cluster count) proportionally so
    that the same structure can be exercised in seconds.  Seeds: 1000+cfg for data and graph,
    2000+cfg for theta_0, 3000+cfg for the sampler.  ``n_groups`` (planted configs) deals the
    clusters greedily into that many size-balanced groups.  ``paper_graph`` (planted configs) keeps the graph
    directed, k out-edges per point in rank order with inverse-rank weights (Section 3.1, Eq. 7), instead of the
    symmetrised unit-weight graph; a cross-cluster replacement may then repeat a neighbour of the row."""
    c = dict(_CONFIGS[cfg])
    n = max(64, int(round(c["n"] * scale)))
    name = f"config{cfg}" + ("" if scale == 1.0 else f"@{scale:g}")
    if c["kind"] == "gmm":
        comps = c["comps"]
        X, comp = gmm_points(n, c["dim"], comps, c["mean_var"], 1000 + cfg, mix=c["mix"],
                             interleave=(cfg == 1), device=device)
        nb = exact_knn(X, c["k"])
        row_ptr, col_idx = knn_lists_to_symmetric_csr(n, nb)
        w = Workload(name=name, n=n, row_ptr=row_ptr, col_idx=col_idx, cluster_of=comp, n_clusters=comps,
                     theta0=init_embedding(n, 2000 + cfg, device=device), n_neg=c["s"], noise_count=c["M"],
                     n_epochs=c["T"], lr0=1.0, seed=3000 + cfg, out_nbrs=nb, X=X, k=c["k"])
        return w
    R = max(2, int(round(c["clusters"] * scale)))
    pg = planted_knn_graph(n, R, c["k"], c["cross"], 1000 + cfg, device=device)
    group = None
    if c.get("own_group"):
        group = torch.arange(R, dtype=torch.int32, device=device)
    if n_groups is not None:
        group = torch.from_numpy(balanced_groups(pg["sizes"], n_groups)).to(device)
    if paper_graph:
        pg["row_ptr"], pg["col_idx"] = directed_rank_csr(pg["out_nbrs"])
        name += "+directed-rank"
    return Workload(name=name, n=n, row_ptr=pg["row_ptr"], col_idx=pg["col_idx"], cluster_of=pg["cluster_of"], weights=None,
                    inverse_rank_weights=paper_graph,
                    n_clusters=R, theta0=init_embedding(n, 2000 + cfg, device=device), n_neg=c["s"],
                    noise_count=c["M"], n_epochs=c["T"], lr0=1.0, seed=3000 + cfg, cluster_group=group,
                    out_nbrs=pg["out_nbrs"], k=c["k"])


def balanced_groups(sizes: np.ndarray, n_groups: int) -> np.ndarray:
    """Greedy size-balanced dealing of clusters to groups (largest cluster first, always to the
    lightest group).  Returns int32 [n_clusters]."""
    load = np.zeros(n_groups, dtype=np.int64)
    out = np.empty(len(sizes), dtype=np.int32)
    for r in np.argsort(-np.asarray(sizes), kind="stable"):
        gsel = int(np.argmin(load))
        out[r] = gsel
        load[gsel] += int(sizes[r])
    return out


# --------------------------------------------------------------------------
# small random problems for unit tests
# --------------------------------------------------------------------------
def random_symmetric_graph(n: int, avg_deg: float, seed: int):
    """Erdos-Renyi-like symmetric graph without self loops, every row non-empty.
    Returns numpy (row_ptr int32, col_idx int32)."""
    rng = np.random.default_rng(seed)
    p = min(1.0, avg_deg / max(1, n - 1))
    a = rng.random((n, n)) < p
    a = np.triu(a, 1)
    for i in range(n):                       # make sure nobody is isolated
        if not a[i].any() and not a[:, i].any():
            j = (i + 1 + int(rng.integers(0, n - 1))) % n
            a[min(i, j), max(i, j)] = True
    a = a | a.T
    row_ptr = np.zeros(n + 1, dtype=np.int32)
    row_ptr[1:] = np.cumsum(a.sum(1))
    col_idx = np.nonzero(a)[1].astype(np.int32)
    return row_ptr, col_idx
