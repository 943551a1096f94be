"""CPU oracle for one NOMAD Projection epoch -- TEST INFRASTRUCTURE, NOT PRODUCT.

Plain, slow, literal Python/numpy in float64.  It exists so that the HIP library
can be checked against something written independently from the paper.  Only
tests, the smoke check and the benchmark's CPU-baseline leg may import it; it
imports nothing from the HIP package and shares no code with it.

What it computes, in the paper's order and notation (arxiv 2505.15511):

  * Cauchy kernel q(a,b) = 1/(1+|a-b|^2)                               -- Eq. 1
  * NOMAD loss: for a head i and each of its graph edges ij,
      l_ij = -log( q(ij) / (q(ij) + Mtilde_i + Mcal_ij) )              -- Eq. 4
      Mtilde_i = |M| * sum_{r in Rtilde_i} p(m in r) q(theta_i, mu_r)  -- Eq. 5
      Mcal_ij  = the noise-sample sum over the cells that are not
                 approximated, estimated from s sampled negatives       -- Eq. 6
    averaged over heads with p(j|i) as edge weights (uniform head marginal,
    Section 3.3).  With no approximated cell this is the InfoNC-t-SNE loss (Eq. 2).
  * mu_r = mean embedding of cell r, p(m in r) = n_r/n under the uniform noise
    distribution over tails (Section 3.3).
  * the gradient of that sampled loss w.r.t. every embedding row it touches
    (head, tail, sampled negatives), with the sample indices and mu held fixed.
  * SGD with a learning rate annealed linearly to zero (Section 3.4).

Readings where the paper is silent (each one is listed in the design notes):
  - p(j|i) is the row-normalised edge weight (unit weights -> 1/deg_i);
  - one epoch = one full-batch step over all heads, each directed edge drawing s fresh
    negatives; the step uses n * grad(L) so lr0 is in per-point units;
  - negatives: Philox4x32-10, counter (lo32(e), hi32(e), t, slot>>2), key (lo32(seed),
    hi32(seed)), word slot&3, index = high word of x * n_loc(i); no rejection;
  - opt-in pooled sampler (a variant, not the paper's i.i.d. noise samples): blocks of
    pool_block consecutive CSR positions share a pool of pool_size uniformly drawn points and
    16 bits of the per-edge Philox words pick a pool entry per slot (see negatives());
  - opt-in pooled sampler with distinct picks (pool_mode = 1; the other pooled variant, see negatives_distinct()):
    the s negatives of one edge sit in s different, independently drawn pool lines, so they are exactly i.i.d.
    uniform over the points as Section 3.1 defines the noise samples of an edge; only negatives of different
    edges of a block are dependent;
  - the cells approximated for head i are those whose group differs from the group of
    i's own cluster; negatives are drawn from the points of i's own group (ascending
    index order) and weighted by omega_i = |M| * (n_loc(i)/n) / s;
  - mu is a constant of the epoch (no gradient through it);
  - eta_t = lr0 * (1 - t/T);
  - optional minibatches: batches_per_epoch = B sequential sub-steps over consecutive head ranges, all with
    eta_t and the cell means of the start of the epoch (see epoch()).

parity status: every function here is pinned by tests/test_oracle_*.py (closed forms,
finite differences, brute force, invariants, Philox known answers).  Absolute embedding
quality against the paper's figures is *parity unpinned*: the paper prints no value for
any workload that can be rebuilt offline.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional

import numpy as np

# Philox4x32 constants of the published algorithm (Salmon et al., SC'11).
_PHILOX_M0 = 0xD2511F53
_PHILOX_M1 = 0xCD9E8D57
_PHILOX_W0 = 0x9E3779B9
_PHILOX_W1 = 0xBB67AE85
_MASK32 = 0xFFFFFFFF


def philox4x32_10(counter, key):
    """Philox4x32 with 10 rounds on Python integers.  counter: 4 words, key: 2 words."""
    c0, c1, c2, c3 = (int(x) & _MASK32 for x in counter)
    k0, k1 = (int(x) & _MASK32 for x in key)
    for _ in range(10):
        p0 = _PHILOX_M0 * c0
        p1 = _PHILOX_M1 * c2
        hi0, lo0 = p0 >> 32, p0 & _MASK32
        hi1, lo1 = p1 >> 32, p1 & _MASK32
        c0, c1, c2, c3 = (hi1 ^ c1 ^ k0) & _MASK32, lo1, (hi0 ^ c3 ^ k1) & _MASK32, lo0
        k0 = (k0 + _PHILOX_W0) & _MASK32
        k1 = (k1 + _PHILOX_W1) & _MASK32
    return (c0, c1, c2, c3)


def philox4x32_10_array(c0, c1, c2, c3, k0, k1):
    """Same generator on numpy arrays of counters (uint64 arithmetic, one shared key)."""
    c0 = np.asarray(c0, dtype=np.uint64); c1 = np.asarray(c1, dtype=np.uint64)
    c2 = np.asarray(c2, dtype=np.uint64); c3 = np.asarray(c3, dtype=np.uint64)
    c0, c1, c2, c3 = np.broadcast_arrays(c0, c1, c2, c3)
    k0 = int(k0) & _MASK32
    k1 = int(k1) & _MASK32
    m32 = np.uint64(_MASK32)
    s32 = np.uint64(32)
    for _ in range(10):
        p0 = np.uint64(_PHILOX_M0) * c0
        p1 = np.uint64(_PHILOX_M1) * c2
        hi0, lo0 = p0 >> s32, p0 & m32
        hi1, lo1 = p1 >> s32, p1 & m32
        c0, c1, c2, c3 = (hi1 ^ c1 ^ np.uint64(k0)), lo1, (hi0 ^ c3 ^ np.uint64(k1)), lo0
        k0 = (k0 + _PHILOX_W0) & _MASK32
        k1 = (k1 + _PHILOX_W1) & _MASK32
    return c0, c1, c2, c3


@dataclasses.dataclass
class Problem:
    """Inputs of the epoch path: a kNN digraph in CSR, a partition into clusters (cells),
    an optional grouping of cells, and the sampling / schedule parameters."""

    n: int
    row_ptr: np.ndarray                       # int [n+1]
    col_idx: np.ndarray                       # int [E]
    cluster_of: np.ndarray                    # int [n]
    n_clusters: int
    n_neg: int                                # s
    noise_count: float                        # |M|   (<= 0 means "= s")
    seed: int = 0
    n_epochs: int = 1                         # T
    lr0: float = 1.0
    weights: Optional[np.ndarray] = None      # [E] or None = unit
    cluster_group: Optional[np.ndarray] = None  # [n_clusters] or None = one group
    pool_size: int = 0                        # pooled sampler: points per pool (0 = i.i.d. per-edge sampler)
    pool_block: int = 0                       # pooled sampler: consecutive CSR positions that share a pool
    batches_per_epoch: int = 1                # B: sequential sub-steps of an epoch over consecutive head ranges
    pool_mode: int = 0                        # pooled sampler: 0 = 16-bit picks, consecutive blocks; 1 = distinct picks,
                                              # interleaved blocks (negatives_distinct); 2 = the same with the pools' lines
                                              # dealt from a permutation (stratified_line_start)
    pool_line: int = 1                        # pool_mode 1: consecutive points per pool line (a power of two)
    pool_segment: int = 64                    # pool_mode 1: consecutive CSR positions dealt to a block together (a power
                                              # of two >= 64 that divides pool_block; = pool_block: consecutive blocks)
    inverse_rank_weights: bool = False        # p(j|i) from the position of j in i's row (Eq. 7) instead of `weights`
    sampled_far_field: bool = False           # opt-in: Eq. 5's sum over approximated cells estimated from the samples
    mean_gradient: bool = False               # opt-in: the gradient also flows through the cell means mu_r(theta)

    def __post_init__(self):
        self.row_ptr = np.asarray(self.row_ptr, dtype=np.int64)
        self.col_idx = np.asarray(self.col_idx, dtype=np.int64)
        self.cluster_of = np.asarray(self.cluster_of, dtype=np.int64)
        if self.inverse_rank_weights:
            assert self.weights is None, "either explicit weights or the rank model"
            self.weights = rank_model_weights(self.row_ptr)
        if self.weights is not None:
            self.weights = np.asarray(self.weights, dtype=np.float32)
        if self.cluster_group is not None:
            self.cluster_group = np.asarray(self.cluster_group, dtype=np.int64)
        if self.noise_count <= 0:
            self.noise_count = float(self.n_neg)
        assert (self.pool_size == 0) == (self.pool_block == 0), "pool_size and pool_block go together"
        assert self.pool_size == 0 or self.cluster_group is None, "the pooled sampler needs a single population"
        assert self.pool_mode in (0, 1, 2) and (self.pool_mode == 0 or self.pool_size > 0), "pool_mode 1 and 2 need a pool"
        if self.pool_mode in (1, 2):
            P_, l_ = self.pool_size, self.pool_line
            assert P_ >= 2 and P_ & (P_ - 1) == 0 and P_ <= 4096, "distinct picks: the pool size is a power of two, 2..4096"
            assert l_ >= 1 and l_ & (l_ - 1) == 0 and P_ % l_ == 0 and self.n_neg <= P_ // l_, "lines: a power of two, s <= lines"
            g_ = self.pool_segment
            assert g_ >= 64 and g_ & (g_ - 1) == 0 and self.pool_block % g_ == 0, "blocks are whole segments; segments a power of two >= 64"
            assert self.batches_per_epoch == 1, "distinct picks: one step per epoch"
        else:
            assert self.pool_line == 1, "pool lines belong to pool_mode 1"
        assert not (self.sampled_far_field and self.pool_size), "sampled far field and pooled sampler do not combine"
        assert not (self.sampled_far_field and self.mean_gradient), "gradient through the means needs the exact far field"
        assert not (self.mean_gradient and self.batches_per_epoch > 1), "sub-steps hold the means of the epoch start constant"

    @property
    def n_edges(self) -> int:
        return int(self.row_ptr[-1])

    @classmethod
    def from_workload(cls, w: dict, **over):
        d = dict(n=w["n"], row_ptr=w["row_ptr"], col_idx=w["col_idx"], cluster_of=w["cluster_of"],
                 n_clusters=w["n_clusters"], n_neg=w["n_neg"], noise_count=w["noise_count"], seed=w["seed"],
                 n_epochs=w["n_epochs"], lr0=w["lr0"], weights=w.get("weights"),
                 cluster_group=w.get("cluster_group"), pool_size=w.get("pool_size", 0), pool_block=w.get("pool_block", 0),
                 pool_mode=w.get("pool_mode", 0), pool_line=w.get("pool_line", 1), pool_segment=w.get("pool_segment", 64),
                 inverse_rank_weights=w.get("inverse_rank_weights", False),
                 batches_per_epoch=w.get("batches_per_epoch", 1), sampled_far_field=w.get("sampled_far_field", False),
                 mean_gradient=w.get("mean_gradient", False))
        d.update(over)
        return cls(**d)


def cauchy(a, b) -> float:
    """q(a,b) = 1/(1+|a-b|^2)  (Eq. 1)."""
    dx = float(a[0]) - float(b[0])
    dy = float(a[1]) - float(b[1])
    return 1.0 / (1.0 + dx * dx + dy * dy)


def edge_probabilities(P: Problem) -> np.ndarray:
    """p(j|i) for every CSR edge: the row-normalised weight (unit weights -> 1/deg_i)."""
    E = P.n_edges
    p = np.zeros(E, dtype=np.float64)
    for i in range(P.n):
        a, b = int(P.row_ptr[i]), int(P.row_ptr[i + 1])
        if b == a:
            continue
        if P.weights is None:
            p[a:b] = 1.0 / (b - a)
        else:
            w = P.weights[a:b].astype(np.float64)
            p[a:b] = w / w.sum()
    return p


def cluster_stats(P: Problem, theta: np.ndarray):
    """Cell sizes n_r, cell masses p(m in r) = n_r/n, and cell means mu_r of theta."""
    R = P.n_clusters
    counts = np.zeros(R, dtype=np.int64)
    sums = np.zeros((R, 2), dtype=np.float64)
    th = np.asarray(theta, dtype=np.float64)
    for i in range(P.n):
        r = int(P.cluster_of[i])
        counts[r] += 1
        sums[r] += th[i]
    mu = np.zeros((R, 2), dtype=np.float64)
    nz = counts > 0
    mu[nz] = sums[nz] / counts[nz, None]
    return counts, counts / float(P.n), mu


def local_sets(P: Problem):
    """group_of_point [n] and, per group, the ascending array of its points (the sampling
    population N_i of every head in that group)."""
    if P.cluster_group is None:
        gop = np.zeros(P.n, dtype=np.int64)
    else:
        gop = P.cluster_group[P.cluster_of]
    members = {}
    for g in np.unique(gop):
        members[int(g)] = np.nonzero(gop == g)[0].astype(np.int64)
    return gop, members


def mean_field(P: Problem, theta: np.ndarray, p_r: np.ndarray, mu: np.ndarray):
    """A_i = sum_{r in Rtilde_i} p_r q(theta_i, mu_r) (so that Mtilde_i = |M| A_i, Eq. 5) and
    B_i = sum_{r in Rtilde_i} p_r q(theta_i, mu_r)^2 (theta_i - mu_r), its derivative factor."""
    n = P.n
    A = np.zeros(n, dtype=np.float64)
    B = np.zeros((n, 2), dtype=np.float64)
    if P.cluster_group is None or P.sampled_far_field:
        return A, B
    th = np.asarray(theta, dtype=np.float64)
    grp = P.cluster_group
    for i in range(n):
        gi = grp[P.cluster_of[i]]
        for r in range(P.n_clusters):
            if grp[r] == gi or p_r[r] == 0.0:
                continue
            q = cauchy(th[i], mu[r])
            A[i] += p_r[r] * q
            B[i] += p_r[r] * q * q * (th[i] - mu[r])
    return A, B


def pool_of_block(P: Problem, beta: int, t: int) -> np.ndarray:
    """Pooled sampler: the pool_size points shared by the CSR positions of block beta in epoch t.
    Entry u is picked by word u & 3 of Philox(counter (beta, 0xFFFFFFFF, t, u >> 2)) (the second
    counter word keeps this stream apart from the per-edge one, whose second word is hi32(e) = 0)."""
    k0, k1 = P.seed & _MASK32, (P.seed >> 32) & _MASK32
    pool = np.zeros(P.pool_size, dtype=np.int64)
    for u in range(P.pool_size):
        words = philox4x32_10((beta & _MASK32, _MASK32, t, u >> 2), (k0, k1))
        pool[u] = (words[u & 3] * P.n) >> 32
    return pool


# Second and third counter words of the two Philox streams of a pool block (the per-edge stream of the i.i.d.
# sampler has hi32(e) = 0 in that place).
_POOL_ENTRY_STREAM = 0xFFFFFFFF
_POOL_PICK_STREAM = 0xFFFFFFFE


def distinct_pool_layout(P: Problem):
    """Pooled sampler with distinct picks: how the CSR positions are dealt to pool blocks.  The positions are cut
    into segments of g = pool_segment; with Q = pool_block / g segments per block there are NB = ceil(NS / Q) blocks
    for NS segments, and segment sigma belongs to block sigma mod NB: a block is made of Q segments spread evenly
    over the whole edge list, so the edges that share a pool come from Q different neighbourhoods of the graph
    (g = pool_block: one segment per block, i.e. blocks of consecutive positions).
    Returns (NB, block(e), rank(e)): rank(e) = g (sigma div NB) + (e mod g) numbers a block's positions."""
    E, g = P.n_edges, P.pool_segment
    NS = (E + g - 1) // g
    Q = P.pool_block // g
    NB = max(1, (NS + Q - 1) // Q)
    return NB, (lambda e: (e // g) % NB), (lambda e: g * ((e // g) // NB) + (e % g))


def distinct_pool_entry(P: Problem, beta: int, t: int, u: int) -> int:
    """Point behind entry u of the pool of block beta in epoch t.  The pool is L = pool_size / pool_line lines of
    pool_line consecutive points (cyclically: the point after n-1 is 0); entry u is point number u div L of line
    u mod L; line gamma starts at a_gamma = floor(x n / 2^32), x = word gamma & 3 of
    Philox(counter (beta, 0xFFFFFFFF, t, gamma >> 2)).  Every entry is uniform over the points (a uniform start
    shifted by a constant, modulo n), entries of different lines are independent."""
    L = P.pool_size // P.pool_line
    gamma, o = u % L, u // L
    if P.pool_mode == 2:
        return (stratified_line_start(P, beta, t, gamma) + o) % P.n
    k0, k1 = P.seed & _MASK32, (P.seed >> 32) & _MASK32
    x = philox4x32_10((beta & _MASK32, _POOL_ENTRY_STREAM, t, gamma >> 2), (k0, k1))[gamma & 3]
    return (((x * P.n) >> 32) + o) % P.n


_POOL_KEY_STREAM = 0xFFFFFFFD


def stratified_keys(P: Problem, t: int):
    """Per-epoch constants of the stratified pools (pool_mode = 2): three odd multipliers A_k, three increments C_k and
    a shift r_t uniform over the points, from two Philox calls with counters (0, 0xFFFFFFFD, t, 0) and (1, 0xFFFFFFFD, t, 0)."""
    k0, k1 = P.seed & _MASK32, (P.seed >> 32) & _MASK32
    w = philox4x32_10((0, _POOL_KEY_STREAM, t, 0), (k0, k1)) + philox4x32_10((1, _POOL_KEY_STREAM, t, 0), (k0, k1))
    return (w[0] | 1, w[2] | 1, w[4] | 1), (w[1], w[3], w[5]), (w[6] * P.n) >> 32


def stratified_line_permutation(x: int, n_lines: int, A, C) -> int:
    """A keyed bijection of 0 .. n_lines-1: on b = max(1, ceil(log2 n_lines)) bits, three rounds of
    x <- (A_k x + C_k) mod 2^b; x <- x xor (x >> max(1, b // 2)) (each a bijection of the b-bit numbers), repeated
    until the value is below n_lines (cycle walking keeps it a bijection of the smaller range)."""
    b = max(1, (n_lines - 1).bit_length())
    mask, sh = (1 << b) - 1, max(1, b // 2)
    while True:
        for k in range(3):
            x = (A[k] * x + C[k]) & mask
            x ^= x >> sh
        if x < n_lines:
            return x


def stratified_line_start(P: Problem, beta: int, t: int, gamma: int) -> int:
    """First point of line gamma of block beta's pool in epoch t (pool_mode = 2).  The n points form NL = ceil(n / l)
    lines of l = pool_line consecutive points; the lines an epoch's pools consist of are dealt from a permutation:
    block beta's line gamma is line number pi_t((beta L + gamma) mod NL), shifted cyclically by r_t:
    start = (l pi_t(.) + r_t) mod n.  Every line of points is then used by the same number of pools of an epoch
    (to within one), instead of a Poisson-distributed number: what a point receives as a negative over an epoch
    fluctuates as little as with independent draws per edge.  Every start is still uniform over the points (r_t is);
    the lines of one pool are distinct, i.e. drawn without replacement."""
    L = P.pool_size // P.pool_line
    NL = (P.n + P.pool_line - 1) // P.pool_line
    A, C, r = stratified_keys(P, t)
    return (P.pool_line * stratified_line_permutation((beta * L + gamma) % NL, NL, A, C) + r) % P.n


def distinct_picks(P: Problem, beta: int, rank: int, t: int):
    """The s pool entries of the position with rank `rank` in block beta.  One 32-bit word W per edge: word
    (rank >> 10) & 3 of Philox(counter (beta, 0xFFFFFFFE, t, (rank & 1023) + 1024 (rank >> 12))), so that one call
    serves four positions 1024 apart.  With lg = log2(pool_size): first entry u_0 = the top lg bits of W, stride
    c = 2 (bits 1 .. lg-1 of W) + 1 (odd), slot k takes entry (u_0 + k c) mod pool_size.  An odd stride visits
    s <= L different residues modulo the number of lines L (a power of two), so the s picks lie in s different
    lines."""
    k0, k1 = P.seed & _MASK32, (P.seed >> 32) & _MASK32
    call = (rank & 1023) + 1024 * (rank >> 12)
    W = philox4x32_10((beta & _MASK32, _POOL_PICK_STREAM, t, call), (k0, k1))[(rank >> 10) & 3]
    lg = P.pool_size.bit_length() - 1
    u0 = W >> (32 - lg)
    c = 2 * ((W >> 1) & (P.pool_size // 2 - 1)) + 1
    return [(u0 + k * c) % P.pool_size for k in range(P.n_neg)]


def negatives_distinct(P: Problem, t: int, e_begin: int, e_end: int) -> np.ndarray:
    """Pooled sampler with distinct picks (pool_mode = 1): m[e, k] = the point behind pool entry distinct_picks()[k] of
    the pool of e's block.  The s negatives of an edge come from s different lines whose starts are independent
    uniform draws, hence they are i.i.d. uniform over the points: the noise samples of one edge are exactly those
    of Section 3.1; negatives of different edges of a block share lines and are dependent."""
    _, block, rank = distinct_pool_layout(P)
    out = np.zeros((e_end - e_begin, P.n_neg), dtype=np.int64)
    for e in range(e_begin, e_end):
        beta = block(e)
        for k, u in enumerate(distinct_picks(P, beta, rank(e), t)):
            out[e - e_begin, k] = distinct_pool_entry(P, beta, t, u)
    return out


def negatives(P: Problem, t: int, e_begin: int = 0, e_end: Optional[int] = None) -> np.ndarray:
    """Sampled negative indices m[e, slot] for the CSR edges e_begin..e_end-1 of epoch t.

    i.i.d. sampler (the paper's |M| i.i.d. noise samples per edge, Section 3.1/3.3): word slot & 3 of
    Philox(counter (lo32 e, hi32 e, t, slot >> 2)) picks a point of the head's population.
    Pooled sampler (opt-in variant): slot k picks entry u = (x16 * pool_size) >> 16 of the pool shared
    by the edge's block of pool_block CSR positions, x16 = 16-bit half k & 1 of word (k >> 1) & 3 of
    Philox(counter (lo32 e, hi32 e, t, k >> 3)).  Each negative is still uniform over the points,
    negatives of one block are no longer independent.
    Sampled far field (opt-in variant): the i.i.d. sampler with every head's population = all n points."""
    if e_end is None:
        e_end = P.n_edges
    s = P.n_neg
    out = np.zeros((e_end - e_begin, s), dtype=np.int64)
    if s == 0 or e_end == e_begin:
        return out
    if P.pool_mode in (1, 2):
        return negatives_distinct(P, t, e_begin, e_end)
    e = np.arange(e_begin, e_end, dtype=np.uint64)
    k0, k1 = P.seed & _MASK32, (P.seed >> 32) & _MASK32
    if P.pool_size > 0:
        pools = {}
        for call in range((s + 7) // 8):
            words = philox4x32_10_array(e & np.uint64(_MASK32), e >> np.uint64(32), np.uint64(t), np.uint64(call), k0, k1)
            for k in range(8 * call, min(s, 8 * call + 8)):
                x16 = (words[(k >> 1) & 3] >> np.uint64(16 * (k & 1))) & np.uint64(0xFFFF)
                for idx in range(e_end - e_begin):
                    beta = (e_begin + idx) // P.pool_block
                    if beta not in pools:
                        pools[beta] = pool_of_block(P, beta, t)
                    out[idx, k] = pools[beta][(int(x16[idx]) * P.pool_size) >> 16]
        return out
    gop, members = local_sets(P)
    head = np.searchsorted(P.row_ptr, np.arange(e_begin, e_end), side="right") - 1
    for blk in range((s + 3) // 4):
        words = philox4x32_10_array(e & np.uint64(_MASK32), e >> np.uint64(32), np.uint64(t), np.uint64(blk), k0, k1)
        for lane in range(4):
            slot = 4 * blk + lane
            if slot >= s:
                break
            x = words[lane]
            for idx in range(e_end - e_begin):
                pop = np.arange(P.n) if P.sampled_far_field else members[int(gop[head[idx]])]
                u = (int(x[idx]) * len(pop)) >> 32
                out[idx, slot] = pop[u]
    return out


def omega(P: Problem) -> np.ndarray:
    """Weight of one sampled negative of head i: |M| * (n_loc(i)/n) / s, which makes the
    sample sum an unbiased estimate of the exact-cell noise term (Eq. 6)."""
    gop, members = local_sets(P)
    w = np.zeros(P.n, dtype=np.float64)
    if P.n_neg == 0:
        return w
    for g, pop in members.items():
        w[gop == g] = P.noise_count * (len(pop) / float(P.n)) / P.n_neg
    if P.sampled_far_field:       # every head samples all points
        w[:] = P.noise_count / P.n_neg
    return w


def _as_positions(theta) -> np.ndarray:
    """The product's embeddings are fp32; a float64 array is taken as it is so that the
    finite-difference checks can perturb below fp32 resolution."""
    theta = np.asarray(theta)
    if theta.dtype == np.float64:
        return theta
    return theta.astype(np.float32).astype(np.float64)


def loss_and_grad(P: Problem, theta: np.ndarray, t: int, want_grad: bool = True, mu_fixed=None, head_range=None):
    """Sampled NOMAD loss L_t(theta) (Eq. 4, uniform head marginal) and g = grad_theta(n * L_t)
    with the negatives of epoch index t.  Returns (L, g [n,2]).  ``mu_fixed`` replaces the cell
    means (the gradient holds them constant; a finite-difference check must do the same).
    ``head_range`` = (begin, end) keeps only the terms of the heads begin..end-1 (one sub-step of a
    minibatch epoch); the terms of all ranges of a partition add up to the full loss and gradient.

    Sampled far field (opt-in variant of Eq. 5): a negative m drawn from all points whose cell r is approximated
    for the head (another group) enters through the cell mean, q(theta_i, mu_r), and receives no force (the means
    are constants of the epoch); a negative of the head's own group enters as itself.  With m uniform over the
    points, E[(|M|/s) sum_k q_k] = |M| sum_{r in Rtilde} p_r q(theta_i, mu_r) + (|M|/n) sum_{m in own group}
    q(theta_i, theta_m): Eq. 5 plus the expectation of the sampled term of Eq. 6, with no sum over the cells.

    Gradient through the means (opt-in; the default holds the means constant): mu_r = (1/n_r) sum_{l in r} theta_l, so
    every member l of an approximated cell r also receives (1/n_r) d(n L)/d mu_r, with
    d(n L)/d mu_r = sum_{i: r in Rtilde_i} sum_{e in row i} p_e (|M| p_r / S_e) 2 q(theta_i, mu_r)^2 (theta_i - mu_r).
    Not defined together with ``mu_fixed`` or a head range whose means come from elsewhere: the means are those
    of ``theta``."""
    th = _as_positions(theta)
    n, s, Mn = P.n, P.n_neg, float(P.noise_count)
    pe = edge_probabilities(P)
    _, p_r, mu = cluster_stats(P, th)
    if mu_fixed is not None:
        mu = np.asarray(mu_fixed, dtype=np.float64)
    A, B = mean_field(P, th, p_r, mu)
    neg = negatives(P, t)
    om = omega(P)
    g = np.zeros((n, 2), dtype=np.float64)
    G_mu = np.zeros((P.n_clusters, 2), dtype=np.float64)      # d(n L)/d mu_r, used with mean_gradient
    total = 0.0
    h0, h1 = (0, n) if head_range is None else head_range
    grp = P.cluster_group

    def through_mean(i, m):
        """sampled far field: is negative m of head i replaced by the mean of its cell?"""
        return P.sampled_far_field and grp is not None and grp[P.cluster_of[m]] != grp[P.cluster_of[i]]

    for i in range(h0, h1):
        for e in range(int(P.row_ptr[i]), int(P.row_ptr[i + 1])):
            j = int(P.col_idx[e])
            d_ij = th[i] - th[j]
            q_ij = 1.0 / (1.0 + d_ij @ d_ij)
            q_im = np.zeros(s)
            where = []
            for kap in range(s):
                m = int(neg[e, kap])
                where.append(mu[P.cluster_of[m]] if through_mean(i, m) else th[m])
                q_im[kap] = cauchy(th[i], where[kap])
            S = q_ij + Mn * A[i] + om[i] * q_im.sum()
            total += pe[e] * (-math.log(q_ij) + math.log(S))
            if not want_grad:
                continue
            a_e = 2.0 * pe[e] * q_ij * (1.0 - q_ij / S)
            g[i] += a_e * d_ij
            g[j] -= a_e * d_ij
            for kap in range(s):
                m = int(neg[e, kap])
                d_im = th[i] - where[kap]
                b = 2.0 * pe[e] * om[i] * q_im[kap] ** 2 / S
                g[i] -= b * d_im
                if not through_mean(i, m):
                    g[m] += b * d_im
            g[i] -= 2.0 * pe[e] * Mn * B[i] / S
            if P.mean_gradient and grp is not None:
                for r in range(P.n_clusters):
                    if grp[r] != grp[P.cluster_of[i]] and p_r[r] > 0.0:
                        q = cauchy(th[i], mu[r])
                        G_mu[r] += pe[e] * (Mn * p_r[r] / S) * 2.0 * q * q * (th[i] - mu[r])
    if P.mean_gradient and want_grad:
        counts = np.bincount(P.cluster_of, minlength=P.n_clusters)
        for l in range(n):
            g[l] += G_mu[P.cluster_of[l]] / counts[P.cluster_of[l]]
    return total / n, g


def learning_rate(P: Problem, t: int) -> float:
    """eta_t = lr0 * (1 - t/T): linear decay towards zero (Section 3.4)."""
    return P.lr0 * (1.0 - t / float(P.n_epochs))


def batch_ranges(P: Problem):
    """Head ranges of the B = batches_per_epoch sub-steps of an epoch: floor(n b / B) .. floor(n (b+1) / B)."""
    B = max(1, int(P.batches_per_epoch))
    return [(P.n * b // B, P.n * (b + 1) // B) for b in range(B)]


def epoch(P: Problem, theta: np.ndarray, t: int):
    """One epoch.  With B = batches_per_epoch = 1: one full-batch step.  With B > 1 (a reading of the paper's
    "approximates the expectation over heads via random sampling", Section 3.3): B sequential sub-steps, sub-step
    b over the heads of batch_ranges()[b], each evaluated at the current theta with the cell means of the start
    of the epoch and followed by theta <- fp32(theta - eta_t g_b).  Returns (theta_next fp32, g of the last
    sub-step fp64, sum of the sub-steps' loss terms)."""
    th32 = np.asarray(theta, dtype=np.float32).copy()
    _, _, mu0 = cluster_stats(P, _as_positions(th32))
    eta = learning_rate(P, t)
    total, g = 0.0, np.zeros((P.n, 2))
    for (h0, h1) in batch_ranges(P):
        L, g = loss_and_grad(P, th32, t, mu_fixed=mu0, head_range=(h0, h1))
        total += L
        th32 = (_as_positions(th32) - eta * g).astype(np.float32)
    return th32, g, total


def inverse_rank_weights(k: int) -> np.ndarray:
    """Inverse-rank edge model (Eq. 7) read with 1-based ranks rho = 1..k and a k-term
    normaliser so that it is a distribution: p(rho) = exp(1/rho) / sum_{rho'=1..k} exp(1/rho')."""
    w = np.exp(1.0 / np.arange(1, k + 1, dtype=np.float64))
    return w / w.sum()


def rank_model_weights(row_ptr) -> np.ndarray:
    """Per-edge weights of a graph whose rows list a head's neighbours in ascending distance: the edge at position
    rho = 1..k_i of row i gets inverse_rank_weights(k_i)[rho - 1] (Eq. 7 with the row's own length k_i)."""
    row_ptr = np.asarray(row_ptr, dtype=np.int64)
    out = np.zeros(int(row_ptr[-1]), dtype=np.float64)
    for i in range(len(row_ptr) - 1):
        a, b = int(row_ptr[i]), int(row_ptr[i + 1])
        if b > a:
            out[a:b] = inverse_rank_weights(b - a)
    return out


def neighbourhood_preservation(nbrs_a: np.ndarray, nbrs_b: np.ndarray) -> float:
    """Mean overlap of two k-neighbour lists per point (Section 4): (1/n) sum_i |A_i & B_i| / k."""
    k = nbrs_a.shape[1]
    tot = 0
    for a, b in zip(nbrs_a, nbrs_b):
        tot += len(set(a.tolist()) & set(b.tolist()))
    return tot / (k * len(nbrs_a))
