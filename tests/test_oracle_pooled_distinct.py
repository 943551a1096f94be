"""Pins for the pooled sampler with distinct picks (pool_mode = 1): what makes it different from the other pooled
variant is a statement about distributions, so the pins are statistical and structural: the negatives of one edge
are i.i.d. uniform over the points (collision rate 1/n, uniform pairs, the exact expectation of the InfoNC-t-SNE loss
of Eq. 2 by enumeration), lines and blocks have the stated structure, both implementations agree."""
import itertools
import math

import numpy as np
import pytest

from oracle import nomad_oracle as po
from paper_2505_15511_amd.workloads import random_symmetric_graph
from tests.oracle_impls import IMPLS

BOTH = pytest.mark.parametrize("impl", ["py", "c"])


def _problem(n, seed, s, P, G, line, deg=6.0, segment=64):
    row_ptr, col = random_symmetric_graph(n, deg, seed)
    return dict(n=n, row_ptr=row_ptr, col_idx=col, cluster_of=np.zeros(n, int), n_clusters=1, n_neg=s, noise_count=float(s),
                seed=(seed << 33) | 5, pool_size=P, pool_block=G, pool_mode=1, pool_line=line, pool_segment=segment)


def test_both_implementations_draw_the_same_negatives():
    for (n, s, P, G, line, seg) in ((300, 5, 64, 128, 4, 64), (1000, 3, 16, 64, 1, 64), (777, 7, 256, 1024, 16, 256), (50, 4, 8, 192, 2, 64),
                                    (5000, 5, 2048, 4096, 16, 1024), (40, 2, 4, 8192, 2, 128), (3000, 5, 64, 2048, 8, 2048)):
        kw = _problem(n, 3, s, P, G, line, segment=seg)
        a, b = IMPLS["py"](**kw), IMPLS["c"](**kw)
        for t in (0, 6):
            ma = a.negatives(t, 0, min(len(kw["col_idx"]), 3000))
            assert np.array_equal(ma, b.negatives(t, 0, min(len(kw["col_idx"]), 3000)))
            assert ma.min() >= 0 and ma.max() < n
        assert not np.array_equal(a.negatives(0, 0, 500), a.negatives(1, 0, 500))          # the epoch enters the counters


def test_picks_of_an_edge_lie_in_different_lines_and_blocks_are_interleaved():
    kw = _problem(2000, 4, 5, 64, 256, 8)
    P = po.Problem(**kw)
    NB, block, rank = po.distinct_pool_layout(P)
    E = P.n_edges
    assert NB == -(-(-(-E // 64)) // 4)                                      # four segments of 64 positions per block
    L = 64 // 8
    for e in range(0, E, 37):
        picks = po.distinct_picks(P, block(e), rank(e), 2)
        assert len(set(picks)) == 5 and len({u % L for u in picks}) == 5     # distinct entries, distinct lines
        assert all(0 <= u < 64 for u in picks)
    # a block's positions: 64 consecutive ones, then the next 64 a whole round of blocks further on
    assert block(0) == block(63) == block(64 * NB) and block(64) == 1 and rank(64 * NB + 3) == 64 + 3
    ranks = sorted(rank(e) for e in range(E) if block(e) == 2)
    assert ranks == list(range(len(ranks))) and len(ranks) <= 256
    # one segment per block: blocks of consecutive positions
    Pc = po.Problem(**dict(kw, pool_segment=256))
    NBc, blockc, rankc = po.distinct_pool_layout(Pc)
    assert NBc == -(-E // 256) and all(blockc(e) == e // 256 and rankc(e) == e % 256 for e in range(0, E, 101))
    # the entries of a line are cyclically consecutive points; entries of the pool are what the negatives consist of
    pool = [po.distinct_pool_entry(P, 2, 1, u) for u in range(64)]
    for g in range(L):
        line = [pool[o * L + g] for o in range(8)]
        assert [(x - line[0]) % P.n for x in line] == list(range(8))
    neg = po.negatives(P, 1)
    mine = np.array([block(e) == 2 for e in range(E)])
    assert set(neg[mine].reshape(-1).tolist()) <= set(pool)
    assert len(set(neg[~mine].reshape(-1).tolist()) - set(pool)) > 100      # other blocks have other pools


@BOTH
def test_two_negatives_of_one_edge_collide_at_rate_one_over_n(impl):
    """i.i.d. uniform draws coincide with probability 1/n.  The other pooled variant lets two slots of an edge take the
    same pool entry (probability 1/P on top); with distinct lines that cannot happen."""
    n = 40
    for line in (1, 4):
        kw = _problem(n, 5, 4, 16, 64, line, deg=8.0)
        O = IMPLS[impl](**kw)
        hits = pairs = 0
        for t in range(400 if impl == "c" else 25):
            m = O.negatives(t)
            for a, b in itertools.combinations(range(4), 2):
                hits += int((m[:, a] == m[:, b]).sum())
                pairs += len(m)
        rate, se = hits / pairs, math.sqrt((1 / n) / pairs)
        assert abs(rate - 1 / n) < 5 * se * 3                               # pairs of one epoch share lines: wide margin
    kw0 = dict(kw, pool_mode=0, pool_line=1)
    O0 = IMPLS["c"](**kw0)
    m = np.concatenate([O0.negatives(t) for t in range(200)])
    assert (m[:, 0] == m[:, 1]).mean() > 1 / n + 0.5 / 16                    # the 16-bit picks do collide inside the pool


def test_pairs_of_negatives_of_one_edge_are_uniform_over_all_pairs_of_points():
    """chi-square of (m_0, m_1) over the n^2 cells, and of a single slot over the n points, with lines of four points
    (a pair inside one line would pile up next to the diagonal)."""
    n = 12
    kw = _problem(n, 6, 3, 16, 64, 4, deg=5.0)
    O = IMPLS["c"](**kw)
    E = len(kw["col_idx"])
    cells = np.zeros((n, n))
    single = np.zeros(n)
    T = 6000
    for t in range(T):
        m = O.negatives(t)[::7]          # thin out: edges of a block share lines, the statistic wants independent draws
        np.add.at(cells, (m[:, 0], m[:, 2]), 1)
        np.add.at(single, m[:, 1], 1)
    N = cells.sum()
    chi2 = ((cells - N / n ** 2) ** 2 / (N / n ** 2)).sum()
    dof = n * n - 1
    assert chi2 < dof + 6 * math.sqrt(2 * dof) * 4                           # dependent edges inflate the variance a little
    off = np.array([cells[a, (a + d) % n] for a in range(n) for d in (1, 2, 3)]).mean()
    assert abs(off - N / n ** 2) < 0.05 * N / n ** 2                         # neighbours in index are not favoured
    chi1 = ((single - single.sum() / n) ** 2 / (single.sum() / n)).sum()
    assert chi1 < (n - 1) + 6 * math.sqrt(2 * (n - 1)) * 4


def test_expected_sampled_loss_is_the_infonc_loss_of_eq_2():
    """With M = s i.i.d. uniform negatives per edge the expectation of the sampled loss over the sampler IS Eq. 2,
    whose expectation over M can be enumerated on five points.  Negatives that are not independent inside an edge
    miss it (the other pooled variant, same pool size, is off by several standard errors)."""
    n, M = 5, 2
    row_ptr = np.arange(0, 2 * n + 1, 2)
    col = np.stack([(np.arange(n) - 1) % n, (np.arange(n) + 1) % n], 1).reshape(-1)
    rng = np.random.default_rng(5)
    theta = (np.round(rng.normal(size=(n, 2)) * 0.8 * 1024) / 1024).astype(np.float32)
    th = theta.astype(np.float64)
    q = 1.0 / (1.0 + ((th[:, None, :] - th[None, :, :]) ** 2).sum(-1))
    exact = 0.0
    for i in range(n):
        for e in range(row_ptr[i], row_ptr[i + 1]):
            j = col[e]
            exact += sum(-math.log(q[i, j] / (q[i, j] + q[i, a] + q[i, b])) for a in range(n) for b in range(n)) / n ** 2 / 2
    exact /= n
    kw = dict(n=n, row_ptr=row_ptr, col_idx=col, cluster_of=np.zeros(n, int), n_clusters=1, n_neg=M, noise_count=float(M), seed=99,
              pool_size=4, pool_block=64)
    T = 20000
    O = IMPLS["c"](**kw, pool_mode=1, pool_line=2)
    draws = np.array([O.loss_and_grad(theta, t, want_grad=False)[0] for t in range(T)])
    se = draws.std() / math.sqrt(T)
    assert abs(draws.mean() - exact) < 4 * se and se < 0.004
    O0 = IMPLS["c"](**kw)                      # 16-bit picks from the same four entries: slots coincide a quarter of the time
    draws0 = np.array([O0.loss_and_grad(theta, t, want_grad=False)[0] for t in range(T)])
    assert abs(draws0.mean() - exact) > 6 * draws0.std() / math.sqrt(T)


def test_sample_sum_is_unbiased_for_every_edge():
    """E[(|M|/s) sum_k q(i, m_k)] = |M| (1/n) sum_l q(i, l) for every edge (each negative is uniform over the points)."""
    n = 40
    kw = _problem(n, 23, 4, 8, 64, 2)
    kw["noise_count"] = 6.0
    O = IMPLS["c"](**kw)
    rng = np.random.default_rng(23)
    theta = rng.normal(size=(n, 2))
    head = np.searchsorted(kw["row_ptr"], np.arange(len(kw["col_idx"])), side="right") - 1
    q = 1.0 / (1.0 + ((theta[:, None, :] - theta[None, :, :]) ** 2).sum(-1))
    est = np.zeros(len(head))
    T = 3000
    for t in range(T):
        est += (6.0 / 4) * q[head[:, None], O.negatives(t)].sum(1)
    est /= T
    want = 6.0 * q[head].mean(1)
    assert np.abs(est - want).max() < 0.05 * want.max()
    assert abs((est - want).mean()) < 0.003 * want.mean()


@BOTH
def test_loss_gradient_and_epoch_with_distinct_picks(impl):
    """The sampler only changes which negatives an edge sees: loss and gradient are those of the plain problem evaluated on
    these negatives (finite differences of the loss; the two implementations agree; an epoch is the plain SGD step)."""
    kw = _problem(30, 8, 3, 8, 64, 2)
    kw.update(n_epochs=6, lr0=0.3)
    O = IMPLS[impl](**kw)
    theta = (np.round(np.random.default_rng(8).normal(size=(30, 2)) * 1024) / 1024).astype(np.float32)
    L, g = O.loss_and_grad(theta, 2)
    L2, g2 = IMPLS["py"](**kw).loss_and_grad(theta, 2)
    assert abs(L - L2) < 1e-13 and np.abs(g - g2).max() < 1e-13
    assert np.abs(g.sum(0)).max() < 1e-13                                    # every force is paired
    if impl == "py":
        P = O.P
        th = theta.astype(np.float64)
        fd = np.zeros_like(g)
        for i in range(P.n):
            for c in range(2):
                tp, tm = th.copy(), th.copy()
                tp[i, c] += 1e-6
                tm[i, c] -= 1e-6
                fd[i, c] = P.n * (po.loss_and_grad(P, tp, 2, want_grad=False)[0] - po.loss_and_grad(P, tm, 2, want_grad=False)[0]) / 2e-6
        assert np.abs(fd - g).max() < 1e-7 * max(1.0, np.abs(g).max())
    nxt, g3, _ = O.epoch(theta, 2)
    assert np.array_equal(nxt, (theta.astype(np.float64) - 0.3 * (1 - 2 / 6) * g).astype(np.float32)) and np.array_equal(g3, g)


# ---------------------------------------------------------------- stratified pools (pool_mode = 2)
def _stratified(n, seed, s, P, G, line, segment=64, deg=6.0):
    return dict(_problem(n, seed, s, P, G, line, deg=deg, segment=segment), pool_mode=2)


def test_line_permutation_is_a_bijection_for_every_size_and_key():
    rng = np.random.default_rng(1)
    for NL in (1, 2, 3, 5, 8, 13, 64, 100, 257, 1000, 4097):
        for _ in range(4):
            A = tuple(int(x) | 1 for x in rng.integers(0, 2 ** 32, 3))
            C = tuple(int(x) for x in rng.integers(0, 2 ** 32, 3))
            out = [po.stratified_line_permutation(x, NL, A, C) for x in range(NL)]
            assert sorted(out) == list(range(NL))
    # keys: two Philox calls; the multipliers are odd, the shift lies in the points' range, another epoch gives other keys
    P = po.Problem(**_stratified(300, 3, 3, 16, 64, 2))
    A, C, r = po.stratified_keys(P, 4)
    w = po.philox4x32_10((0, 0xFFFFFFFD, 4, 0), (P.seed & 0xFFFFFFFF, P.seed >> 32)) + po.philox4x32_10((1, 0xFFFFFFFD, 4, 0), (P.seed & 0xFFFFFFFF, P.seed >> 32))
    assert A == (w[0] | 1, w[2] | 1, w[4] | 1) and C == (w[1], w[3], w[5]) and r == (w[6] * 300) >> 32 and 0 <= r < 300
    assert po.stratified_keys(P, 5) != po.stratified_keys(P, 4)


def test_every_line_of_points_serves_the_same_number_of_pools():
    """What the variant is for: over the pools of one epoch every line of points is used floor or ceil(NB L / NL) times, so
    every point is a pool member equally often (independent draws would give a Poisson-distributed number)."""
    for (n, P_, G, line) in ((640, 64, 128, 4), (1000, 16, 64, 1), (784, 256, 1024, 16)):
        kw = _stratified(n, 4, 3, P_, G, line)
        P = po.Problem(**kw)
        NB, _, _ = po.distinct_pool_layout(P)
        L, NL = P_ // line, n // line
        for t in (0, 3):
            members = np.zeros(n, int)
            for beta in range(NB):
                pool = [po.distinct_pool_entry(P, beta, t, u) for u in range(P_)]
                assert len(set(pool)) == P_                                       # the lines of one pool are distinct (n is a multiple of the line)
                for g in range(L):
                    assert [(pool[o * L + g] - pool[g]) % n for o in range(line)] == list(range(line))
                np.add.at(members, pool, 1)
            lo, hi = (NB * L) // NL, -(-(NB * L) // NL)
            assert members.min() >= lo and members.max() <= hi and members.sum() == NB * P_
        iid = po.Problem(**dict(kw, pool_mode=1))
        spread = np.zeros(n, int)
        for beta in range(NB):
            np.add.at(spread, [po.distinct_pool_entry(iid, beta, 0, u) for u in range(P_)], 1)
        assert spread.max() - spread.min() > hi - lo + 1                          # independent draws are not that even


def test_stratified_negatives_are_uniform_over_the_points_and_both_implementations_agree():
    for (n, s, P_, G, line, seg) in ((300, 5, 64, 128, 4, 64), (1000, 3, 16, 64, 1, 64), (777, 7, 256, 1024, 16, 256), (50, 4, 8, 192, 2, 64),
                                     (5000, 5, 2048, 4096, 16, 1024)):
        kw = _stratified(n, 3, s, P_, G, line, segment=seg)
        a, b = IMPLS["py"](**kw), IMPLS["c"](**kw)
        hi = min(len(kw["col_idx"]), 2500)
        for t in (0, 6):
            assert np.array_equal(a.negatives(t, 0, hi), b.negatives(t, 0, hi))
    n = 24
    O = IMPLS["c"](**_stratified(n, 6, 3, 16, 64, 1, deg=5.0))    # lines of one point: no pair of points is ruled out but (a, a)
    single = np.zeros(n)
    pairs = np.zeros((n, n))
    for t in range(6000):
        m = O.negatives(t)[::5]
        np.add.at(single, m[:, 1], 1)
        np.add.at(pairs, (m[:, 0], m[:, 2]), 1)
    chi1 = ((single - single.sum() / n) ** 2 / (single.sum() / n)).sum()
    assert chi1 < (n - 1) + 24 * math.sqrt(2 * (n - 1))                       # every negative is uniform (the shift r_t is)
    # two negatives of an edge lie in different lines: never the same point, every other pair about equally often
    assert np.trace(pairs) == 0
    off = pairs[~np.eye(n, dtype=bool)]
    assert off.min() > 0.6 * off.mean() and off.max() < 1.5 * off.mean()


def test_expected_loss_with_stratified_pools_is_eq_2_with_noise_samples_drawn_without_replacement():
    """Lines of one point: the s negatives of an edge are s different points, (close to) uniform over such tuples, so the
    expectation of the sampled loss is Eq. 2's with the noise samples of an edge drawn without replacement, enumerated here
    on 7 points; the difference to independent draws is of order s^2 / n and vanishes at real sizes."""
    n, M = 7, 2
    row_ptr = np.arange(0, 2 * n + 1, 2)
    col = np.stack([(np.arange(n) - 1) % n, (np.arange(n) + 1) % n], 1).reshape(-1)
    rng = np.random.default_rng(5)
    theta = (np.round(rng.normal(size=(n, 2)) * 0.8 * 1024) / 1024).astype(np.float32)
    th = theta.astype(np.float64)
    q = 1.0 / (1.0 + ((th[:, None, :] - th[None, :, :]) ** 2).sum(-1))
    exact = 0.0
    for i in range(n):
        for e in range(row_ptr[i], row_ptr[i + 1]):
            j = col[e]
            exact += sum(-math.log(q[i, j] / (q[i, j] + q[i, a] + q[i, b])) for a in range(n) for b in range(n) if a != b) / (n * (n - 1)) / 2
    exact /= n
    kw = dict(n=n, row_ptr=row_ptr, col_idx=col, cluster_of=np.zeros(n, int), n_clusters=1, n_neg=M, noise_count=float(M), seed=99,
              pool_size=4, pool_block=64, pool_mode=2, pool_line=1)
    T = 20000
    O = IMPLS["c"](**kw)
    draws = np.array([O.loss_and_grad(theta, t, want_grad=False)[0] for t in range(T)])
    se = draws.std() / math.sqrt(T)
    assert abs(draws.mean() - exact) < 5 * se + 2e-3 * exact       # the keyed permutations are not all permutations: a small allowance
