"""Pins for the oracle's loss, gradient, means and update: closed forms, finite differences,
an independently written brute-force evaluator, exact expectations on tiny graphs and the
invariants the loss has.  Every pin runs on the literal Python oracle and on the C oracle."""
import itertools
import math

import numpy as np
import pytest

from oracle import nomad_oracle as po
from paper_2505_15511_amd.workloads import random_symmetric_graph
from tests.oracle_impls import IMPLS

BOTH = pytest.mark.parametrize("impl", ["py", "c"])


def _ring(n):
    row_ptr = np.arange(0, 2 * n + 1, 2)
    col = np.stack([(np.arange(n) - 1) % n, (np.arange(n) + 1) % n], 1).reshape(-1)
    return row_ptr, col


def _grid_theta(n, seed, scale=1.0):
    """Positions on a 2^-10 grid so that they, and +-2^-8 steps from them, are exact in fp32."""
    rng = np.random.default_rng(seed)
    return (np.round(rng.normal(size=(n, 2)) * scale * 1024) / 1024).astype(np.float32)


def _random_problem(n, seed, groups=True, weights=True, s=3, M=4.0, n_clusters=5):
    row_ptr, col = random_symmetric_graph(n, 4.0, seed)
    rng = np.random.default_rng(seed + 1)
    kw = dict(n=n, row_ptr=row_ptr, col_idx=col, cluster_of=rng.integers(0, n_clusters, n), n_clusters=n_clusters,
              n_neg=s, noise_count=M, seed=seed * 77 + 5)
    kw["cluster_of"][:n_clusters] = np.arange(n_clusters)        # no empty cluster
    if weights:
        kw["weights"] = rng.uniform(0.2, 2.0, size=len(col)).astype(np.float32)
    if groups:
        kw["cluster_group"] = rng.integers(0, 3, n_clusters)
        kw["cluster_group"][:3] = [0, 1, 2]
    return kw


# ---------------------------------------------------------------- P1: coincident points
@BOTH
def test_all_points_coincident_gives_log_one_plus_M_and_zero_force(impl):
    n, s = 40, 5
    row_ptr, col = random_symmetric_graph(n, 5.0, 3)
    O = IMPLS[impl](n=n, row_ptr=row_ptr, col_idx=col, cluster_of=np.zeros(n, int), n_clusters=1, n_neg=s,
                    noise_count=s, seed=1)
    theta = np.full((n, 2), 0.375, dtype=np.float32)
    L, g = O.loss_and_grad(theta, 0)
    assert abs(L - math.log(6.0)) < 1e-14          # every q is 1: l = -log(1/(1+5))
    assert abs(L - 1.791759469228055) < 1e-14
    assert np.abs(g).max() == 0.0


# ---------------------------------------------------------------- P2: two points
def _two_point(impl, seed, s=5, d=1.0):
    O = IMPLS[impl](n=2, row_ptr=[0, 1, 2], col_idx=[1, 0], cluster_of=[0, 0], n_clusters=1, n_neg=s,
                    noise_count=s, seed=seed)
    theta = np.array([[0.0, 0.0], [d, 0.0]], dtype=np.float32)
    return O, theta


@BOTH
def test_two_points_closed_form_for_any_sample(impl):
    """n=2, edges 0<->1 at distance d: with c_e of the s negatives of edge e falling on the other
    point, S_e = q + (s-c_e) + c_e q, l_e = -log q + log S_e and the head of e is pushed by
    2 q d (s-c_e)/S_e along the edge, its tail by the opposite."""
    s, d = 5, 0.75
    q = 1.0 / (1.0 + d * d)
    for seed in range(6):
        O, theta = _two_point(impl, seed, s, d)
        neg = O.negatives(2)
        L, g = O.loss_and_grad(theta, 2)
        c0 = int((neg[0] == 1).sum())
        c1 = int((neg[1] == 0).sum())
        S0, S1 = q + (s - c0) + c0 * q, q + (s - c1) + c1 * q
        assert abs(L - 0.5 * (2 * -math.log(q) + math.log(S0) + math.log(S1))) < 1e-14
        f0 = 2 * q * d * (s - c0) / S0           # edge 0->1: d_01 = (-d, 0)
        f1 = 2 * q * d * (s - c1) / S1           # edge 1->0: d_10 = (+d, 0)
        gx0 = -f0 - f1
        assert abs(g[0, 0] - gx0) < 1e-14 and abs(g[1, 0] + gx0) < 1e-14
        assert g[0, 1] == 0.0 and g[1, 1] == 0.0


@BOTH
def test_two_points_all_negatives_on_self(impl):
    """The worked case d=1, s=5 with every negative equal to the head itself: L = log 11 and
    |g_0| = 20/11 (each directed edge contributes 10/11)."""
    found = None
    for seed in range(20000):
        k = (seed & 0xFFFFFFFF, seed >> 32)
        w0 = po.philox4x32_10((0, 0, 0, 0), k) + po.philox4x32_10((0, 0, 0, 1), k)
        w1 = po.philox4x32_10((1, 0, 0, 0), k) + po.philox4x32_10((1, 0, 0, 1), k)
        # edge 0 (head 0) wants index 0: top bit clear; edge 1 (head 1) wants index 1: top bit set
        if all(x < 2 ** 31 for x in w0[:5]) and all(x >= 2 ** 31 for x in w1[:5]):
            found = seed
            break
    assert found is not None
    O, theta = _two_point(impl, found, 5, 1.0)
    assert np.array_equal(O.negatives(0), [[0] * 5, [1] * 5])
    L, g = O.loss_and_grad(theta, 0)
    assert abs(L - math.log(11.0)) < 1e-14
    assert abs(L - 2.3978952727983707) < 1e-14
    assert abs(abs(g[0, 0]) - 20.0 / 11.0) < 1e-14
    assert g[0, 0] < 0 < g[1, 0]                  # descent (theta -= eta g) pulls the two together
    assert np.allclose(g[0], -g[1], atol=1e-15)


# ---------------------------------------------------------------- P3: no negatives
@BOTH
def test_no_negatives_no_means_is_degenerate(impl):
    n = 30
    row_ptr, col = random_symmetric_graph(n, 4.0, 5)
    O = IMPLS[impl](n=n, row_ptr=row_ptr, col_idx=col, cluster_of=np.zeros(n, int), n_clusters=1, n_neg=0,
                    noise_count=3.0, seed=1)
    L, g = O.loss_and_grad(_grid_theta(n, 1), 0)
    assert abs(L) < 1e-15 and np.abs(g).max() < 1e-15


# ---------------------------------------------------------------- P4: finite differences
def test_gradient_matches_finite_differences_python():
    """Central differences of the loss in float64 with the samples and the cell means held
    fixed; covers head, tail, negative and mean-field terms, weights and groups."""
    for seed in (1, 2):
        kw = _random_problem(24, seed)
        P = po.Problem(**kw)
        rng = np.random.default_rng(seed)
        theta = rng.normal(size=(P.n, 2))
        _, _, mu = po.cluster_stats(P, theta)
        _, g = po.loss_and_grad(P, theta, 1, mu_fixed=mu)
        h = 1e-6
        fd = np.zeros_like(g)
        for i in range(P.n):
            for c in range(2):
                tp, tm = theta.copy(), theta.copy()
                tp[i, c] += h
                tm[i, c] -= h
                Lp, _ = po.loss_and_grad(P, tp, 1, want_grad=False, mu_fixed=mu)
                Lm, _ = po.loss_and_grad(P, tm, 1, want_grad=False, mu_fixed=mu)
                fd[i, c] = P.n * (Lp - Lm) / (2 * h)
        assert np.abs(fd - g).max() < 1e-7 * max(1.0, np.abs(g).max())
        assert np.abs(g).max() > 1e-2


def test_gradient_matches_finite_differences_c():
    """Same check on the C oracle, which takes fp32 positions: five-point central differences
    with a step of 2^-8 on grid positions, so that every perturbed value is exact in fp32."""
    kw = _random_problem(20, 4)
    O = IMPLS["c"](**kw)
    theta = _grid_theta(O.n, 9, scale=0.75)
    _, _, mu = O.cluster_stats(theta)
    _, g = O.loss_and_grad(theta, 3, mu_fixed=mu)
    h = 2.0 ** -8
    fd = np.zeros_like(g)
    for i in range(O.n):
        for c in range(2):
            vals = []
            for k in (-2, -1, 1, 2):
                tt = theta.copy()
                tt[i, c] += np.float32(k * h)
                vals.append(O.loss_and_grad(tt, 3, want_grad=False, mu_fixed=mu)[0])
            fd[i, c] = O.n * (vals[0] - 8 * vals[1] + 8 * vals[2] - vals[3]) / (12 * h)
    assert np.abs(fd - g).max() < 2e-7 * max(1.0, np.abs(g).max())


@BOTH
def test_c_and_python_gradients_agree(impl):
    kw = _random_problem(30, 6)
    theta = _grid_theta(30, 6)
    L0, g0 = IMPLS["py"](**kw).loss_and_grad(theta, 5)
    L1, g1 = IMPLS[impl](**kw).loss_and_grad(theta, 5)
    assert abs(L0 - L1) < 1e-13 and np.abs(g0 - g1).max() < 1e-13


# ---------------------------------------------------------------- P5: brute force
def _brute_force_loss(kw, theta, neg):
    """Written separately from the oracle: dictionary of edges, explicit loops over cells and
    samples, cell means from python lists."""
    n = kw["n"]
    th = [(float(x), float(y)) for x, y in np.asarray(theta, dtype=np.float64)]
    edges = {}
    for i in range(n):
        for e in range(int(kw["row_ptr"][i]), int(kw["row_ptr"][i + 1])):
            w = 1.0 if kw.get("weights") is None else float(kw["weights"][e])
            edges[(i, int(kw["col_idx"][e]), e)] = w
    rowsum = {}
    for (i, _, _), w in edges.items():
        rowsum[i] = rowsum.get(i, 0.0) + w
    cells = {}
    for i in range(n):
        cells.setdefault(int(kw["cluster_of"][i]), []).append(i)
    grp = kw.get("cluster_group")
    group = (lambda r: 0) if grp is None else (lambda r: int(grp[r]))
    s, M = kw["n_neg"], float(kw["noise_count"])

    def q(a, b):
        return 1.0 / (1.0 + (a[0] - b[0]) ** 2 + (a[1] - b[1]) ** 2)

    total = 0.0
    for (i, j, e), w in edges.items():
        gi = group(int(kw["cluster_of"][i]))
        mtilde, nloc = 0.0, 0
        for r, pts in cells.items():
            if group(r) == gi:
                nloc += len(pts)
                continue
            mu = (sum(th[p][0] for p in pts) / len(pts), sum(th[p][1] for p in pts) / len(pts))
            mtilde += M * (len(pts) / n) * q(th[i], mu)
        mcal = 0.0
        for kap in range(s):
            mcal += (M * (nloc / n) / s) * q(th[i], th[int(neg[e][kap])])
        qij = q(th[i], th[j])
        total += (w / rowsum[i]) * -math.log(qij / (qij + mtilde + mcal))
    return total / n


@BOTH
@pytest.mark.parametrize("groups,weights", [(False, False), (True, False), (True, True)])
def test_loss_matches_brute_force(impl, groups, weights):
    kw = _random_problem(18, 11, groups=groups, weights=weights)
    O = IMPLS[impl](**kw)
    theta = _grid_theta(18, 3)
    neg = O.negatives(4)
    L, _ = O.loss_and_grad(theta, 4, want_grad=False)
    assert abs(L - _brute_force_loss(kw, theta, neg)) < 1e-13


# ---------------------------------------------------------------- P6: exact expectations
def _exact_infonc(theta, row_ptr, col, M):
    """Eq. 2 with the expectation over M i.i.d. uniform negatives enumerated exactly."""
    n = len(theta)
    q = 1.0 / (1.0 + ((theta[:, None, :] - theta[None, :, :]) ** 2).sum(-1))
    tot = 0.0
    for i in range(n):
        deg = row_ptr[i + 1] - row_ptr[i]
        for e in range(row_ptr[i], row_ptr[i + 1]):
            j = col[e]
            acc = 0.0
            for tup in itertools.product(range(n), repeat=M):
                acc += -math.log(q[i, j] / (q[i, j] + sum(q[i, m] for m in tup)))
            tot += acc / (n ** M) / deg
    return tot / n


def test_sample_mean_of_loss_converges_to_exact_infonc_expectation():
    """With nothing approximated the oracle's loss, averaged over many sample draws, is the
    InfoNC-t-SNE loss (Eq. 2) whose expectation over negatives can be enumerated on 5 points."""
    n, M = 5, 2
    row_ptr, col = _ring(n)
    theta = _grid_theta(n, 5, scale=0.8)
    exact = _exact_infonc(theta.astype(np.float64), row_ptr, col, M)
    O = IMPLS["c"](n=n, row_ptr=row_ptr, col_idx=col, cluster_of=np.zeros(n, int), n_clusters=1, n_neg=M,
                   noise_count=M, seed=99)
    draws = np.array([O.loss_and_grad(theta, t, want_grad=False)[0] for t in range(4000)])
    se = draws.std() / math.sqrt(len(draws))
    assert abs(draws.mean() - exact) < 4 * se
    assert se < 0.01


@BOTH
def test_singleton_cells_give_the_exact_upper_bound_and_it_dominates_infonc(impl):
    """Every point its own cell and its own group: the approximated term is |M| (1/n) sum_{l != i} q(il)
    exactly (a one-point cell equals its mean) and the sampled remainder is |M|/n (self, q = 1), so
    the loss is the Jensen bound of the proof of Theorem 1 in closed form -- and it must not be
    smaller than the exact InfoNC-t-SNE loss."""
    n, M = 5, 2
    row_ptr, col = _ring(n)
    for seed in (1, 2, 3):
        theta = _grid_theta(n, seed, scale=1.5)
        O = IMPLS[impl](n=n, row_ptr=row_ptr, col_idx=col, cluster_of=np.arange(n), n_clusters=n, n_neg=3,
                        noise_count=M, seed=seed, cluster_group=np.arange(n))
        L, _ = O.loss_and_grad(theta, 0, want_grad=False)
        th = theta.astype(np.float64)
        q = 1.0 / (1.0 + ((th[:, None, :] - th[None, :, :]) ** 2).sum(-1))
        bound = 0.0
        for i in range(n):
            for e in range(row_ptr[i], row_ptr[i + 1]):
                j = col[e]
                bound += 0.5 * -math.log(q[i, j] / (q[i, j] + M * q[i].mean()))
        bound /= n
        assert abs(L - bound) < 1e-14
        assert bound >= _exact_infonc(th, row_ptr, col, M) - 1e-12


# ---------------------------------------------------------------- P7: Taylor step is second order
@BOTH
def test_mean_approximation_error_is_second_order_in_cell_radius(impl):
    n = 41
    row_ptr, col = _ring(n)
    cluster_of = np.array([0] + [1] * 40)
    ang = np.arange(40) * (2 * math.pi / 40)
    errs = []
    for rho in (0.5, 0.25, 0.125):
        theta = np.zeros((n, 2))
        theta[1:, 0] = 4.0 + rho * np.cos(ang)
        theta[1:, 1] = 1.0 + rho * np.sin(ang)
        theta = theta.astype(np.float32)
        O = IMPLS[impl](n=n, row_ptr=row_ptr, col_idx=col, cluster_of=cluster_of, n_clusters=2, n_neg=1,
                        noise_count=1.0, seed=0, cluster_group=[0, 1])
        A, _ = O.mean_field(theta)
        th = theta.astype(np.float64)
        exact = (40.0 / n) * np.mean(1.0 / (1.0 + ((th[0] - th[1:]) ** 2).sum(1)))
        errs.append(abs(A[0] - exact))
    assert 3.6 < errs[0] / errs[1] < 4.4 and 3.6 < errs[1] / errs[2] < 4.4


# ---------------------------------------------------------------- P8: reduction to InfoNC-t-SNE
@BOTH
def test_one_group_equals_no_groups_bit_for_bit(impl):
    kw = _random_problem(25, 8, groups=False)
    theta = _grid_theta(25, 8)
    La, ga = IMPLS[impl](**kw).loss_and_grad(theta, 2)
    kw["cluster_group"] = np.full(kw["n_clusters"], 3)
    Lb, gb = IMPLS[impl](**kw).loss_and_grad(theta, 2)
    assert La == Lb and np.array_equal(ga, gb)


# ---------------------------------------------------------------- P9: invariants
@BOTH
def test_forces_cancel_and_loss_is_rigid_motion_invariant(impl):
    kw = _random_problem(30, 12, groups=False)
    O = IMPLS[impl](**kw)
    theta = _grid_theta(30, 12)
    L, g = O.loss_and_grad(theta, 7)
    assert np.abs(g.sum(0)).max() < 1e-13                      # every force is paired
    shift = theta + np.float32([0.5, -0.25])                     # exact in fp32 on the grid
    L2, g2 = O.loss_and_grad(shift, 7)
    assert abs(L - L2) < 1e-14 and np.abs(g - g2).max() < 1e-13
    rot = np.stack([-theta[:, 1], theta[:, 0]], 1)               # rotation by 90 degrees, exact
    L3, g3 = O.loss_and_grad(rot, 7)
    assert abs(L - L3) < 1e-14
    assert np.abs(np.stack([-g[:, 1], g[:, 0]], 1) - g3).max() < 1e-13
    mir = theta * np.float32([-1.0, 1.0])                        # mirror image
    L4, g4 = O.loss_and_grad(mir, 7)
    assert abs(L - L4) < 1e-14 and np.abs(g * [-1.0, 1.0] - g4).max() < 1e-13


@BOTH
def test_grouped_loss_is_translation_invariant_and_means_are_constants(impl):
    kw = _random_problem(30, 13, groups=True)
    O = IMPLS[impl](**kw)
    theta = _grid_theta(30, 13)
    L, g = O.loss_and_grad(theta, 1)
    L2, g2 = O.loss_and_grad(theta + np.float32([2.0, 1.0]), 1)
    assert abs(L - L2) < 1e-13 and np.abs(g - g2).max() < 1e-12
    assert np.abs(g.sum(0)).max() > 1e-3        # means take force but are not moved: no pairing


# ---------------------------------------------------------------- P10: sample weight is unbiased
def test_sample_weight_makes_the_negative_term_unbiased():
    n = 40
    kw = _random_problem(n, 21, groups=True, s=4, M=6.0)
    O = IMPLS["c"](**kw)
    theta = _grid_theta(n, 21).astype(np.float64)
    gop = np.asarray(kw["cluster_group"])[kw["cluster_of"]]
    om = po.omega(po.Problem(**kw))
    head = np.searchsorted(kw["row_ptr"], np.arange(len(kw["col_idx"])), side="right") - 1
    q = 1.0 / (1.0 + ((theta[:, None, :] - theta[None, :, :]) ** 2).sum(-1))
    est = np.zeros(len(head))
    T = 3000
    for t in range(T):
        neg = O.negatives(t)
        est += om[head] * q[head[:, None], neg].sum(1)
    est /= T
    want = np.array([6.0 * q[i, gop == gop[i]].sum() / n for i in head])
    assert np.abs(est - want).max() < 0.05 * want.max()
    assert abs((est - want).mean()) < 0.003 * want.mean()


def test_pooled_sampler_keeps_the_negative_term_unbiased():
    """Pool entries are uniform over the points and the pick ignores the pool, so the pooled sample sum has the
    same expectation as the i.i.d. one: |M| (1/n) sum_l q_il for every edge."""
    n = 40
    kw = _random_problem(n, 23, groups=False, s=4, M=6.0)
    O = IMPLS["c"](**kw, pool_size=8, pool_block=16)
    theta = _grid_theta(n, 23).astype(np.float64)
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


# ---------------------------------------------------------------- means, update, weights, metric
@BOTH
def test_cluster_statistics(impl):
    n = 50
    kw = _random_problem(n, 31, n_clusters=7)
    O = IMPLS[impl](**kw)
    theta = _grid_theta(n, 31)
    counts, p_r, mu = O.cluster_stats(theta)
    assert counts.sum() == n and abs(p_r.sum() - 1.0) < 1e-15
    for r in range(7):
        sel = kw["cluster_of"] == r
        assert counts[r] == sel.sum()
        assert np.allclose(mu[r], theta[sel].astype(np.float64).mean(0), atol=1e-15)
    # the count-weighted mean of the cell means is the global mean
    assert np.allclose((p_r[:, None] * mu).sum(0), theta.astype(np.float64).mean(0), atol=1e-14)


@BOTH
def test_update_is_plain_sgd_with_linear_decay(impl):
    kw = _random_problem(20, 41, groups=False)
    kw.update(n_epochs=8, lr0=0.5)
    O = IMPLS[impl](**kw)
    theta = _grid_theta(20, 41)
    for t, eta in ((0, 0.5), (4, 0.25), (7, 0.0625)):
        _, g = O.loss_and_grad(theta, t)
        nxt, g2, _ = O.epoch(theta, t)
        assert nxt.dtype == np.float32
        assert np.array_equal(nxt, (theta.astype(np.float64) - eta * g).astype(np.float32))
        assert np.array_equal(g, g2)


@BOTH
def test_descent_direction_lowers_the_sampled_loss(impl):
    kw = _random_problem(30, 51, groups=True)
    kw.update(n_epochs=10, lr0=0.05)
    O = IMPLS[impl](**kw)
    theta = _grid_theta(30, 51)
    _, _, mu = O.cluster_stats(theta)
    L0, _ = O.loss_and_grad(theta, 0, want_grad=False, mu_fixed=mu)
    nxt, _, _ = O.epoch(theta, 0)
    L1, _ = O.loss_and_grad(nxt, 0, want_grad=False, mu_fixed=mu)
    assert L1 < L0


def test_inverse_rank_model_is_a_distribution():
    """Eq. 7 read with ranks 1..k and a k-term normaliser."""
    p15, p10 = po.inverse_rank_weights(15), po.inverse_rank_weights(10)
    assert abs(p15.sum() - 1) < 1e-15 and abs(p10.sum() - 1) < 1e-15
    assert abs(p15[0] / p15[-1] - math.exp(1 - 1 / 15)) < 1e-12
    assert abs(p10[0] / p10[-1] - math.exp(1 - 1 / 10)) < 1e-12
    z15 = sum(math.exp(1.0 / r) for r in range(1, 16))
    assert abs(z15 - 19.363821) < 1e-5 and abs(p15[0] - math.e / z15) < 1e-15
    assert abs(p15[0] - 0.140379) < 1e-6
    assert np.all(np.diff(p15) < 0)


def test_paper_graph_workload_and_the_rank_model_of_the_oracle():
    """The directed workload: k out-edges per point in rank order and a flag instead of weights; both oracles then weigh
    position rho of a row of length k_i by the model of Eq. 7 for k_i neighbours, rows of any length."""
    from paper_2505_15511_amd import workloads
    w = workloads.make_config(3, scale=0.003, paper_graph=True)
    d = w.numpy()
    k = w.k
    assert d["weights"] is None and d["inverse_rank_weights"]
    assert np.array_equal(d["row_ptr"], np.arange(w.n + 1) * k)
    assert np.array_equal(d["col_idx"].reshape(w.n, k), w.out_nbrs.numpy())
    assert not np.any(d["col_idx"].reshape(w.n, k) == np.arange(w.n)[:, None])
    sym = workloads.make_config(3, scale=0.003).numpy()
    assert len(sym["col_idx"]) > len(d["col_idx"])          # the benchmark graph adds the transposed edges
    P = po.Problem.from_workload(d)
    assert np.allclose(P.weights.reshape(w.n, k), po.inverse_rank_weights(k)[None, :], rtol=1e-7, atol=0)
    # ragged rows: lengths 3, 0, 1, 2
    rp = np.array([0, 3, 3, 4, 6])
    wr = po.rank_model_weights(rp)
    z3 = math.exp(1.0) + math.exp(0.5) + math.exp(1 / 3)
    assert np.allclose(wr, [math.e / z3, math.exp(0.5) / z3, math.exp(1 / 3) / z3, 1.0, math.e / (math.e + math.exp(0.5)), math.exp(0.5) / (math.e + math.exp(0.5))], atol=1e-15)
    kw = dict(n=4, row_ptr=rp, col_idx=[1, 2, 3, 0, 0, 1], cluster_of=[0, 0, 0, 0], n_clusters=1, n_neg=2, noise_count=2.0, seed=3)
    theta = _grid_theta(4, 5)
    for impl in ("py", "c"):
        a = IMPLS[impl](**kw, inverse_rank_weights=True).loss_and_grad(theta, 0)
        b = IMPLS[impl](**kw, weights=wr.astype(np.float32)).loss_and_grad(theta, 0)
        assert a[0] == b[0] and np.array_equal(a[1], b[1])


def test_neighbourhood_preservation_metric():
    a = np.array([[1, 2, 3], [0, 2, 3], [0, 1, 3], [0, 1, 2]])
    assert po.neighbourhood_preservation(a, a) == 1.0
    b = np.array([[3, 2, 1], [0, 2, 9], [7, 8, 9], [0, 1, 2]])
    assert abs(po.neighbourhood_preservation(a, b) - (3 + 2 + 0 + 3) / 12.0) < 1e-15


# ---------------------------------------------------------------- minibatch epochs
@BOTH
def test_batch_terms_partition_the_full_loss_and_gradient(impl):
    """The head ranges of the sub-steps partition the heads, so at a fixed theta and fixed means their loss terms
    and gradients add up to the full ones (whatever touches a point as tail or negative lands in the batch of the
    edge's head)."""
    n = 40
    kw = _random_problem(n, 41)
    O = IMPLS[impl](**kw)
    theta = _grid_theta(n, 41)
    _, _, mu = O.cluster_stats(theta)
    L, g = O.loss_and_grad(theta, 3, mu_fixed=mu)
    cuts = [0, 7, 7, 19, 33, n]                      # includes an empty range
    parts = [O.loss_and_grad(theta, 3, mu_fixed=mu, head_range=(a, b)) for a, b in zip(cuts[:-1], cuts[1:])]
    assert abs(sum(p[0] for p in parts) - L) < 1e-13
    assert np.abs(sum(p[1] for p in parts) - g).max() < 1e-13
    # a batch only moves points its edges touch: a head outside the range that is nobody's tail or negative stays put
    assert np.all(parts[1][1] == 0) and parts[1][0] == 0.0


@BOTH
def test_minibatch_epoch_is_sequential_sgd_over_head_ranges(impl):
    """epoch() with B sub-steps equals B hand-made steps: gradient of the batch's edges at the current theta with
    the means of the start of the epoch, then theta <- fp32(theta - eta_t g); B = 1 is the full-batch epoch."""
    n, B, t = 30, 4, 2
    kw = _random_problem(n, 43)
    kw.update(n_epochs=5, lr0=0.3)
    O1 = IMPLS[impl](**kw)
    OB = IMPLS[impl](**kw, batches_per_epoch=B)
    theta = _grid_theta(n, 43).astype(np.float32)
    _, _, mu0 = O1.cluster_stats(theta)
    eta = 0.3 * (1 - t / 5)
    th, total = theta.copy(), 0.0
    for b in range(B):
        L, g = O1.loss_and_grad(th, t, mu_fixed=mu0, head_range=(n * b // B, n * (b + 1) // B))
        total += L
        th = (th.astype(np.float64) - eta * g).astype(np.float32)
    th_B, g_B, L_B = OB.epoch(theta, t)
    assert np.array_equal(th_B, th) and np.abs(g_B - g).max() < 1e-15 and abs(L_B - total) < 1e-13
    th_1, g_1, L_1 = O1.epoch(theta, t)
    L_full, g_full = O1.loss_and_grad(theta, t)
    assert np.array_equal(th_1, (theta.astype(np.float64) - eta * g_full).astype(np.float32)) and abs(L_1 - L_full) < 1e-13
    assert not np.array_equal(th_1, th_B)            # the sub-steps see the moved points


def test_minibatch_epochs_agree_between_the_two_implementations():
    kw = _random_problem(60, 47, s=4)
    kw.update(n_epochs=6, lr0=0.2)
    theta = _grid_theta(60, 47).astype(np.float32)
    a = IMPLS["py"](**kw, batches_per_epoch=5).epoch(theta, 1)
    b = IMPLS["c"](**kw, batches_per_epoch=5).epoch(theta, 1)
    assert np.array_equal(a[0], b[0]) and np.abs(a[1] - b[1]).max() < 1e-12 and abs(a[2] - b[2]) < 1e-12


# ---------------------------------------------------------------- single gradient rows, whole training runs
def _problem_with_idle_points(seed, sampled_far_field=False):
    """Grouped, weighted random problem on 48 connected points plus six points without any edge: three of them
    in a cluster of an active group (they move only as sampled negatives) and three in a cluster that is a group
    of its own (no head samples from it: under the exact far field they never move at all)."""
    n_live, n = 48, 54
    kw = _random_problem(n_live, seed, groups=True, weights=True, s=3, M=4.0, n_clusters=5)
    kw["n"] = n
    kw["row_ptr"] = np.concatenate([np.asarray(kw["row_ptr"]), np.full(n - n_live, kw["row_ptr"][-1])])
    kw["cluster_of"] = np.concatenate([np.asarray(kw["cluster_of"]), [0, 0, 0, 5, 5, 5]])
    kw["n_clusters"] = 6
    kw["cluster_group"] = np.concatenate([np.asarray(kw["cluster_group"]), [7]])
    kw["sampled_far_field"] = sampled_far_field
    return kw


@pytest.mark.parametrize("sampled_far_field", [False, True])
def test_single_gradient_rows_equal_the_rows_of_the_full_gradient(sampled_far_field):
    """The C oracle's row-by-row mode (only the edges that touch a wanted point are evaluated) is the reference at
    sizes where the full pass is out of reach; here it is held against the full gradient, whose definition the
    finite-difference and brute-force pins above fix."""
    for seed in (3, 4):
        kw = _problem_with_idle_points(seed, sampled_far_field)
        O = IMPLS["c"](**kw)
        n = kw["n"]
        theta = _grid_theta(n, seed + 60)
        for t in (0, 5):
            _, g = O.loss_and_grad(theta, t)
            neg = O.negatives(t)
            sampled = np.zeros(n, bool)
            sampled[neg.reshape(-1)] = True
            # the idle points of the active cluster are hit as negatives and by nothing else
            assert sampled[48:51].any() and np.abs(g[48:51]).max() > 0
            if not sampled_far_field:
                assert not sampled[51:].any() and np.all(g[51:] == 0.0)     # a group no head belongs to
            for pts in (np.arange(n), np.array([50, 3, 49, 17, 53, 48, 0, 51]), np.array([52]), np.array([11])):
                rows = O.grad_at(theta, t, pts)
                assert rows.shape == (len(pts), 2)
                assert np.abs(rows - g[pts]).max() < 1e-13
        # and against the literal Python oracle, rows picked from its full gradient
        _, g_py = IMPLS["py"](**kw).loss_and_grad(theta, 5)
        pts = np.array([49, 2, 30, 52])
        assert np.abs(O.grad_at(theta, 5, pts) - g_py[pts]).max() < 1e-13


@pytest.mark.parametrize("variant", ["plain", "grouped", "batches", "pooled"])
def test_training_run_is_the_epoch_applied_T_times(variant):
    """oracle_train (the reference of every full-training check) = epochs t = 0..T-1 of the literal Python oracle
    chained through float32 positions, bit for bit; its loss curve is the loss at the start of every epoch."""
    n, T = 36, 5
    kw = _random_problem(n, 71, groups=(variant in ("grouped", "batches")), weights=True, s=3, M=4.0)
    kw.update(n_epochs=T, lr0=0.4)
    if variant == "batches":
        kw["batches_per_epoch"] = 3
    if variant == "pooled":
        kw.update(pool_size=8, pool_block=16)
    theta0 = _grid_theta(n, 72).astype(np.float32)
    O, Opy = IMPLS["c"](**kw), IMPLS["py"](**kw)
    th_c, curve = O.train(theta0, 0, T)
    th, starts = theta0.copy(), []
    for t in range(T):
        starts.append(th.copy())
        th, _, _ = Opy.epoch(th, t)
    assert th_c.dtype == np.float32 and np.array_equal(th_c, th)
    assert not np.array_equal(th_c, theta0)
    if variant != "batches":       # with sub-steps the curve adds terms evaluated at different positions
        for t in range(T):
            assert abs(curve[t] - Opy.loss_and_grad(starts[t], t, want_grad=False)[0]) < 1e-13
    # a run split in two continues where it stopped (epoch indices, not call counts, key the samples and the step)
    half, _ = O.train(theta0, 0, 2)
    rest, _ = O.train(half, 2, T)
    assert np.array_equal(rest, th_c)


def test_mean_field_sums_of_single_heads():
    """The per-head evaluator of Eq. 5's sums (used at sizes where every head's sums are out of reach) against the
    literal Python oracle's sums over all heads, and against the sum written out for one head."""
    kw = _problem_with_idle_points(9)
    n = kw["n"]
    theta = _grid_theta(n, 91)
    A_py, B_py = IMPLS["py"](**kw).mean_field(theta)
    O = IMPLS["c"](**kw)
    heads = np.array([53, 0, 17, 17, 48, 30])
    A, B = O.mean_field_at(theta, heads)
    assert np.abs(A - A_py[heads]).max() < 1e-15 and np.abs(B - B_py[heads]).max() < 1e-15
    assert A.min() > 0
    # head 17 by hand: cells of other groups, weighted by their share of the points, seen through their means
    th = theta.astype(np.float64)
    grp, cl = np.asarray(kw["cluster_group"]), np.asarray(kw["cluster_of"])
    a = 0.0
    for r in range(kw["n_clusters"]):
        if grp[r] == grp[cl[17]]:
            continue
        mu = th[cl == r].mean(0)
        a += (cl == r).sum() / n / (1.0 + ((th[17] - mu) ** 2).sum())
    assert abs(A[2] - a) < 1e-15
    # nothing is approximated without groups, and the sampled far field has no such sums
    kw1 = dict(kw, cluster_group=None)
    assert np.all(IMPLS["c"](**kw1).mean_field_at(theta, heads)[0] == 0)
    assert np.all(IMPLS["c"](**dict(kw, sampled_far_field=True)).mean_field_at(theta, heads)[0] == 0)
