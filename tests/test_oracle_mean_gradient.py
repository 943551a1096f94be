"""Pins for the oracle's opt-in gradient through the cell means (the default holds mu_r constant within an epoch):
finite differences of the loss with the means recomputed from the perturbed positions, the invariances that the loss
has as a function of the positions alone, reduction to the default when no cell is approximated."""
import numpy as np
import pytest

from oracle import nomad_oracle as po
from tests.oracle_impls import IMPLS
from tests.test_oracle_pins import _grid_theta, _random_problem

BOTH = pytest.mark.parametrize("impl", ["py", "c"])


def test_gradient_is_the_derivative_of_the_loss_with_moving_means_python():
    for seed, weights in ((51, True), (52, False)):
        kw = _random_problem(22, seed, groups=True, weights=weights, s=3)
        P = po.Problem(**kw, mean_gradient=True)
        theta = np.random.default_rng(seed).normal(size=(P.n, 2))
        _, g = po.loss_and_grad(P, theta, 1)
        h, fd = 1e-6, np.zeros((P.n, 2))
        for i in range(P.n):
            for c in range(2):
                tp, tm = theta.copy(), theta.copy()
                tp[i, c] += h
                tm[i, c] -= h
                fd[i, c] = P.n * (po.loss_and_grad(P, tp, 1, want_grad=False)[0] - po.loss_and_grad(P, tm, 1, want_grad=False)[0]) / (2 * h)
        assert np.abs(fd - g).max() < 1e-7 * max(1.0, np.abs(g).max()) and np.abs(g).max() > 1e-2
        # the default gradient (means held constant) is not that derivative
        _, g_const = po.loss_and_grad(po.Problem(**kw), theta, 1)
        assert np.abs(fd - g_const).max() > 1e-3


def test_gradient_is_the_derivative_of_the_loss_with_moving_means_c():
    """fp32 positions on a grid, five-point differences with a step that is exact in fp32."""
    kw = _random_problem(20, 53, groups=True, s=3)
    O = IMPLS["c"](**kw, mean_gradient=True)
    theta = _grid_theta(O.n, 53, scale=0.75)
    _, g = O.loss_and_grad(theta, 2)
    h, fd = 2.0 ** -8, np.zeros((O.n, 2))
    for i in range(O.n):
        for c in range(2):
            vals = []
            for k in (-2, -1, 1, 2):
                tt = theta.copy()
                tt[i, c] += np.float32(k * h)
                vals.append(O.loss_and_grad(tt, 2, want_grad=False)[0])
            fd[i, c] = O.n * (vals[0] - 8 * vals[1] + 8 * vals[2] - vals[3]) / (12 * h)
    assert np.abs(fd - g).max() < 2e-7 * max(1.0, np.abs(g).max())


@BOTH
def test_forces_cancel_and_exert_no_torque_once_the_means_move(impl):
    """As a function of the positions alone the loss is invariant under rigid motions: the gradient sums to zero and
    has no net torque.  With the means held constant neither holds (they take force but are not moved)."""
    kw = _random_problem(40, 54, groups=True, s=4)
    theta = _grid_theta(40, 54, scale=1.5)
    _, g = IMPLS[impl](**kw, mean_gradient=True).loss_and_grad(theta, 3)
    th = theta.astype(np.float64)
    assert np.abs(g.sum(0)).max() < 1e-12
    assert abs((th[:, 0] * g[:, 1] - th[:, 1] * g[:, 0]).sum()) < 1e-12
    _, g_const = IMPLS[impl](**kw).loss_and_grad(theta, 3)
    assert np.abs(g_const.sum(0)).max() > 1e-3


@BOTH
def test_without_approximated_cells_nothing_changes(impl):
    kw = _random_problem(30, 55, groups=False, s=3)
    theta = _grid_theta(30, 55)
    (L0, g0), (L1, g1) = IMPLS[impl](**kw).loss_and_grad(theta, 1), IMPLS[impl](**kw, mean_gradient=True).loss_and_grad(theta, 1)
    assert L0 == L1 and np.array_equal(g0, g1)


def test_both_implementations_agree_on_an_epoch():
    kw = _random_problem(50, 56, groups=True, s=3)
    kw.update(n_epochs=10, lr0=0.5, mean_gradient=True)
    theta = _grid_theta(50, 56)
    (t0, g0, L0), (t1, g1, L1) = IMPLS["py"](**kw).epoch(theta, 2), IMPLS["c"](**kw).epoch(theta, 2)
    assert np.array_equal(t0, t1) and np.abs(g0 - g1).max() < 1e-13 and abs(L0 - L1) < 1e-12
