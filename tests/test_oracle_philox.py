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
