"""Pins for the oracle's sampled far field (opt-in variant of Eq. 5: a negative drawn from all points whose cell is
approximated for the head enters through the cell mean): reductions to the pinned plain sampler, a separately
written brute-force evaluator, the expectation it has to have, finite differences.  Both implementations."""
import math

import numpy as np
import pytest

from oracle import nomad_oracle as po
from tests.oracle_impls import IMPLS
from tests.test_oracle_pins import _grid_theta, _random_problem

BOTH = pytest.mark.parametrize("impl", ["py", "c"])


@BOTH
def test_one_group_reduces_to_the_plain_sampler(impl):
    """Nothing is approximated when all cells share a group: same negatives, loss and gradient as without groups."""
    kw = _random_problem(30, 41, groups=False)
    theta = _grid_theta(30, 41)
    plain = IMPLS[impl](**kw)
    far = IMPLS[impl](**kw, cluster_group=np.zeros(kw["n_clusters"], int), sampled_far_field=True)
    assert np.array_equal(plain.negatives(2), far.negatives(2))
    (L0, g0), (L1, g1) = plain.loss_and_grad(theta, 2), far.loss_and_grad(theta, 2)
    assert L0 == L1 and np.array_equal(g0, g1)


@BOTH
def test_negatives_come_from_all_points_whatever_the_groups(impl):
    kw = _random_problem(40, 42, groups=True, s=6)
    no_groups = {k: v for k, v in kw.items() if k != "cluster_group"}
    assert np.array_equal(IMPLS[impl](**kw, sampled_far_field=True).negatives(7), IMPLS[impl](**no_groups).negatives(7))
    assert not np.array_equal(IMPLS[impl](**kw).negatives(7), IMPLS[impl](**no_groups).negatives(7))


def _brute_force(kw, theta, neg):
    """Loss and gradient written separately from the oracle: python lists, explicit loops."""
    n, s, M = kw["n"], kw["n_neg"], float(kw["noise_count"])
    th = [(float(x), float(y)) for x, y in np.asarray(theta, dtype=np.float64)]
    cell = [int(c) for c in kw["cluster_of"]]
    group = [int(g) for g in kw["cluster_group"]]
    mean = {}
    for r in set(cell):
        pts = [p for p in range(n) if cell[p] == r]
        mean[r] = (sum(th[p][0] for p in pts) / len(pts), sum(th[p][1] for p in pts) / len(pts))
    total, g = 0.0, [[0.0, 0.0] for _ in range(n)]
    for i in range(n):
        a, b = int(kw["row_ptr"][i]), int(kw["row_ptr"][i + 1])
        w = [1.0 if kw.get("weights") is None else float(kw["weights"][e]) for e in range(a, b)]
        for e in range(a, b):
            p = w[e - a] / sum(w)
            j = int(kw["col_idx"][e])
            dij = (th[i][0] - th[j][0], th[i][1] - th[j][1])
            qij = 1.0 / (1.0 + dij[0] ** 2 + dij[1] ** 2)
            terms = []
            for k in range(s):
                m = int(neg[e][k])
                far = group[cell[m]] != group[cell[i]]
                x = mean[cell[m]] if far else th[m]
                d = (th[i][0] - x[0], th[i][1] - x[1])
                terms.append((m, far, d, 1.0 / (1.0 + d[0] ** 2 + d[1] ** 2)))
            S = qij + (M / s) * sum(t[3] for t in terms)
            total += p * (math.log(S) - math.log(qij))
            a_e = 2.0 * p * qij * (1.0 - qij / S)
            for c in range(2):
                g[i][c] += a_e * dij[c]
                g[j][c] -= a_e * dij[c]
            for m, far, d, q in terms:
                bk = 2.0 * p * (M / s) * q * q / S
                for c in range(2):
                    g[i][c] -= bk * d[c]
                    if not far:
                        g[m][c] += bk * d[c]
    return total / n, np.array(g)


@BOTH
@pytest.mark.parametrize("weights", [False, True])
def test_loss_and_gradient_match_brute_force(impl, weights):
    kw = _random_problem(22, 43, groups=True, weights=weights, s=4)
    O = IMPLS[impl](**kw, sampled_far_field=True)
    theta = _grid_theta(22, 43, scale=1.5)
    L, g = O.loss_and_grad(theta, 3)
    L0, g0 = _brute_force(kw, theta, O.negatives(3))
    assert abs(L - L0) < 1e-13 and np.abs(g - g0).max() < 1e-13
    far = np.asarray(kw["cluster_group"])[np.asarray(kw["cluster_of"])[O.negatives(3)]]
    head = np.searchsorted(kw["row_ptr"], np.arange(len(kw["col_idx"])), side="right") - 1
    own = np.asarray(kw["cluster_group"])[np.asarray(kw["cluster_of"])[head]]
    assert (far != own[:, None]).any() and (far == own[:, None]).any()      # both kinds of negative occur


def test_sample_sum_has_the_expectation_of_eq5_plus_eq6():
    """(|M|/s) sum_k q(theta_i, x_k), x_k the mean of m's cell when that cell is approximated and theta_m otherwise,
    averages to |M| [sum_{r approximated} p_r q(theta_i, mu_r) + (1/n) sum_{m in own group} q(theta_i, theta_m)]."""
    n, M, s = 40, 6.0, 4
    kw = _random_problem(n, 44, groups=True, s=s, M=M)
    O = IMPLS["c"](**kw, sampled_far_field=True)
    theta = _grid_theta(n, 44, scale=1.5).astype(np.float64)
    cell, grp = np.asarray(kw["cluster_of"]), np.asarray(kw["cluster_group"])
    gop = grp[cell]
    _, p_r, mu = O.cluster_stats(theta.astype(np.float32))
    head = np.searchsorted(kw["row_ptr"], np.arange(len(kw["col_idx"])), side="right") - 1
    q_pt = 1.0 / (1.0 + ((theta[:, None, :] - theta[None, :, :]) ** 2).sum(-1))          # [i, m]
    q_mu = 1.0 / (1.0 + ((theta[:, None, :] - mu[None, :, :]) ** 2).sum(-1))             # [i, r]
    est, T = np.zeros(len(head)), 3000
    for t in range(T):
        neg = O.negatives(t)
        far = gop[neg] != gop[head][:, None]
        est += (M / s) * np.where(far, q_mu[head[:, None], cell[neg]], q_pt[head[:, None], neg]).sum(1)
    est /= T
    want = np.array([M * ((p_r * q_mu[i])[grp != gop[i]].sum() + q_pt[i, gop == gop[i]].sum() / n) for i in head])
    assert np.abs(est - want).max() < 0.05 * want.max()
    assert abs((est - want).mean()) < 0.003 * want.mean()
    # and that is the noise term the exact far field has in expectation: Eq. 5's sum plus Eq. 6's sampled part
    A, _ = IMPLS["c"](**kw).mean_field(theta.astype(np.float32))
    assert np.allclose(want, M * (A[head] + np.array([q_pt[i, gop == gop[i]].sum() / n for i in head])), rtol=1e-12)


def test_singleton_cells_reduce_to_the_plain_loss():
    """Every point its own cell and group: a cell mean is its point, so the loss equals the plain sampler's."""
    n = 25
    kw = _random_problem(n, 45, groups=False, s=5)
    kw.update(cluster_of=np.arange(n), n_clusters=n)
    theta = _grid_theta(n, 45)
    for impl in ("py", "c"):
        L0, _ = IMPLS[impl](**kw).loss_and_grad(theta, 1, want_grad=False)
        L1, g1 = IMPLS[impl](**kw, cluster_group=np.arange(n), sampled_far_field=True).loss_and_grad(theta, 1)
        assert abs(L0 - L1) < 1e-14
        # no negative receives a force (each stands for a cell), so the forces no longer cancel
        assert np.abs(g1.sum(0)).max() > 1e-3


def test_gradient_matches_finite_differences_python():
    kw = _random_problem(24, 46, groups=True, s=3)
    P = po.Problem(**kw, sampled_far_field=True)
    theta = np.random.default_rng(46).normal(size=(P.n, 2))
    _, _, mu = po.cluster_stats(P, theta)
    _, g = po.loss_and_grad(P, theta, 1, mu_fixed=mu)
    h, fd = 1e-6, np.zeros((P.n, 2))
    for i in range(P.n):
        for c in range(2):
            tp, tm = theta.copy(), theta.copy()
            tp[i, c] += h
            tm[i, c] -= h
            fd[i, c] = P.n * (po.loss_and_grad(P, tp, 1, want_grad=False, mu_fixed=mu)[0] -
                              po.loss_and_grad(P, tm, 1, want_grad=False, mu_fixed=mu)[0]) / (2 * h)
    assert np.abs(fd - g).max() < 1e-7 * max(1.0, np.abs(g).max()) and np.abs(g).max() > 1e-2


def test_both_implementations_agree_on_an_epoch_with_sub_steps():
    kw = _random_problem(60, 47, groups=True, s=3)
    kw.update(n_epochs=10, lr0=0.5, batches_per_epoch=3, sampled_far_field=True)
    theta = _grid_theta(60, 47)
    (t0, g0, L0), (t1, g1, L1) = IMPLS["py"](**kw).epoch(theta, 2), IMPLS["c"](**kw).epoch(theta, 2)
    assert np.array_equal(t0, t1) and np.abs(g0 - g1).max() < 1e-13 and abs(L0 - L1) < 1e-12
