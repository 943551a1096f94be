"""Pins for the sampler of the oracle: published known answers, independent implementations,
avalanche, range reduction, uniformity."""
import os

import numpy as np
import pytest

from oracle import c_oracle, nomad_oracle as po
from tests.oracle_impls import IMPLS

HERE = os.path.dirname(os.path.abspath(__file__))


def _kat():
    rows = []
    for line in open(os.path.join(HERE, "golden", "philox4x32_10_kat.txt")):
        line = line.split("#")[0].strip()
        if line:
            w = [int(x, 16) for x in line.split()]
            rows.append((w[0:4], w[4:6], tuple(w[6:10])))
    return rows


@pytest.mark.parametrize("ctr,key,want", _kat())
def test_known_answers(ctr, key, want):
    assert po.philox4x32_10(ctr, key) == want
    assert c_oracle.philox(ctr, key) == want
    got = po.philox4x32_10_array(*[np.array([c]) for c in ctr], key[0], key[1])
    assert tuple(int(g[0]) for g in got) == want


def test_three_implementations_agree_on_random_counters():
    rng = np.random.default_rng(7)
    c = rng.integers(0, 2 ** 32, size=(200, 4), dtype=np.uint64)
    k = rng.integers(0, 2 ** 32, size=2, dtype=np.uint64)
    arr = po.philox4x32_10_array(c[:, 0], c[:, 1], c[:, 2], c[:, 3], int(k[0]), int(k[1]))
    for r in range(200):
        a = po.philox4x32_10(c[r], k)
        assert a == c_oracle.philox(c[r], k)
        assert a == tuple(int(w[r]) for w in arr)


def test_every_input_word_matters():
    base_c, base_k = [5, 0, 3, 1], [11, 22]
    ref = po.philox4x32_10(base_c, base_k)
    for pos in range(4):
        c = list(base_c); c[pos] ^= 1
        out = po.philox4x32_10(c, base_k)
        assert all(o != r for o, r in zip(out, ref))
    for pos in range(2):
        k = list(base_k); k[pos] ^= 1
        out = po.philox4x32_10(base_c, k)
        assert all(o != r for o, r in zip(out, ref))


def _ring(n):
    row_ptr = np.arange(0, 2 * n + 1, 2)
    col = np.stack([(np.arange(n) - 1) % n, (np.arange(n) + 1) % n], 1).reshape(-1)
    return row_ptr, col


@pytest.mark.parametrize("impl", ["py", "c"])
def test_negative_index_is_counter_keyed_multiply_high(impl):
    """m[e,slot] = floor(x * n / 2^32) with x = word slot&3 of Philox(counter=(e,0,t,slot>>2), key=seed)."""
    n, s, seed, t = 1000, 7, (0x1234 << 32) | 0xBEEF, 9
    row_ptr, col = _ring(n)
    O = IMPLS[impl](n=n, row_ptr=row_ptr, col_idx=col, cluster_of=np.zeros(n, int), n_clusters=1, n_neg=s,
                    noise_count=s, seed=seed)
    neg = O.negatives(t)
    assert neg.shape == (2 * n, s)
    for e in (0, 1, 777, 2 * n - 1):
        for slot in range(s):
            w = po.philox4x32_10((e, 0, t, slot >> 2), (seed & 0xFFFFFFFF, seed >> 32))
            assert neg[e, slot] == (w[slot & 3] * n) >> 32
    # sub-range query returns the same rows
    assert np.array_equal(O.negatives(t, 100, 140), neg[100:140])
    # other epoch, other seed => other samples
    assert not np.array_equal(O.negatives(t + 1), neg)


@pytest.mark.parametrize("impl", ["py", "c"])
def test_negatives_drawn_from_own_group_in_ascending_order(impl):
    n, s = 60, 4
    row_ptr, col = _ring(n)
    cluster_of = np.arange(n) % 6            # interleaved clusters
    group = np.array([0, 1, 0, 1, 2, 2])    # three groups of 20 points, none contiguous
    O = IMPLS[impl](n=n, row_ptr=row_ptr, col_idx=col, cluster_of=cluster_of, n_clusters=6, n_neg=s,
                    noise_count=5.0, seed=42, cluster_group=group)
    neg = O.negatives(3)
    gop = group[cluster_of]
    for e in range(2 * n):
        i = e // 2
        pop = np.nonzero(gop == gop[i])[0]
        for slot in range(s):
            w = po.philox4x32_10((e, 0, 3, slot >> 2), (42, 0))
            assert neg[e, slot] == pop[(w[slot & 3] * len(pop)) >> 32]


def test_uniformity_chi_square():
    n, s = 50, 8
    row_ptr, col = _ring(4000)
    O = IMPLS["c"](n=4000, row_ptr=row_ptr, col_idx=col, cluster_of=np.zeros(4000, int), n_clusters=1, n_neg=s,
                   noise_count=s, seed=2024)
    neg = O.negatives(0)
    bins = np.bincount((neg.reshape(-1) * n // 4000), minlength=n).astype(float)
    exp = neg.size / n
    chi2 = ((bins - exp) ** 2 / exp).sum()
    assert chi2 < 100.0      # 49 dof: mean 49, sd 9.9
    # slots are not copies of one another
    assert (neg[:, 0] != neg[:, 1]).mean() > 0.99
    assert (neg[:, 3] != neg[:, 4]).mean() > 0.99


# ------------------------------------------------------------------ pooled sampler (opt-in variant)
@pytest.mark.parametrize("impl", ["py", "c"])
def test_pooled_negative_is_pool_entry_picked_by_the_edge_word(impl):
    """m[e,k] = pool_beta[(x16 * P) >> 16], beta = e // G, x16 = half k&1 of word (k>>1)&3 of
    Philox(counter=(e, 0, t, k>>3)); pool_beta[u] = floor(y * n / 2^32), y = word u&3 of
    Philox(counter=(beta, 0xFFFFFFFF, t, u>>2))."""
    n, s, seed, t, P, G = 1000, 11, (7 << 32) | 99, 4, 48, 128
    row_ptr, col = _ring(n)
    O = IMPLS[impl](n=n, row_ptr=row_ptr, col_idx=col, cluster_of=np.zeros(n, int), n_clusters=1, n_neg=s,
                    noise_count=s, seed=seed, pool_size=P, pool_block=G)
    neg = O.negatives(t)
    key = (seed & 0xFFFFFFFF, seed >> 32)
    for e in (0, 127, 128, 1031, 2 * n - 1):
        for slot in range(s):
            x16 = (po.philox4x32_10((e, 0, t, slot >> 3), key)[(slot >> 1) & 3] >> (16 * (slot & 1))) & 0xFFFF
            u = (x16 * P) >> 16
            y = po.philox4x32_10((e // G, 0xFFFFFFFF, t, u >> 2), key)[u & 3]
            assert neg[e, slot] == (y * n) >> 32
    assert np.array_equal(O.negatives(t, 100, 300), neg[100:300])      # a range that crosses a block boundary
    assert not np.array_equal(O.negatives(t + 1), neg)


def test_pooled_blocks_share_at_most_pool_size_points_and_differ_between_blocks():
    n, s, P, G = 5000, 5, 32, 512
    row_ptr, col = _ring(n)
    O = IMPLS["c"](n=n, row_ptr=row_ptr, col_idx=col, cluster_of=np.zeros(n, int), n_clusters=1, n_neg=s,
                   noise_count=s, seed=5, pool_size=P, pool_block=G)
    neg = O.negatives(0)
    pools = [set(neg[b * G:(b + 1) * G].reshape(-1).tolist()) for b in range(len(neg) // G)]
    assert all(len(p) <= P for p in pools)
    assert all(len(p) >= P - 2 for p in pools)          # 2560 picks among 32 entries hit every entry; entries may coincide
    assert len(pools[0] & pools[1]) <= 2                # independent pools of 32 among 5000 points
    # one entry per pool: every negative of a block is the same point (degenerate case, closed form)
    O1 = IMPLS["c"](n=n, row_ptr=row_ptr, col_idx=col, cluster_of=np.zeros(n, int), n_clusters=1, n_neg=s,
                    noise_count=s, seed=5, pool_size=1, pool_block=G)
    neg1 = O1.negatives(0)
    for b in range(3):
        assert len(set(neg1[b * G:(b + 1) * G].reshape(-1).tolist())) == 1


def test_pool_entries_are_uniform_over_the_points():
    """The pool entries are the only place where points are drawn: chi-square on 500 pools of 64 entries.
    (The pick of an entry does not look at the pool, so every negative inherits this marginal.)"""
    n = 4000
    row_ptr, col = _ring(n)
    P = po.Problem(n=n, row_ptr=row_ptr, col_idx=col, cluster_of=np.zeros(n, int), n_clusters=1, n_neg=5,
                   noise_count=5, seed=77, pool_size=64, pool_block=16)
    draws = np.concatenate([po.pool_of_block(P, beta, 2) for beta in range(500)])
    bins = np.bincount(draws * 50 // n, minlength=50).astype(float)
    exp = draws.size / 50
    assert ((bins - exp) ** 2 / exp).sum() < 100.0      # 49 dof: mean 49, sd 9.9
    assert not np.array_equal(po.pool_of_block(P, 0, 2), po.pool_of_block(P, 0, 3))
    assert not np.array_equal(po.pool_of_block(P, 0, 2), po.pool_of_block(P, 1, 2))
