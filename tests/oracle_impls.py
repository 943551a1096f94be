"""Uniform view of the two oracle implementations (literal Python and plain C) so that every
pin runs on both."""
import numpy as np

from oracle import c_oracle, nomad_oracle as po


class PyOracle:
    name = "py"

    def __init__(self, **kw):
        kw.pop("theta0", None)
        self.P = po.Problem(**kw)
        self.n = self.P.n

    def negatives(self, t, e_begin=0, e_end=None):
        return po.negatives(self.P, t, e_begin, e_end)

    def cluster_stats(self, theta):
        return po.cluster_stats(self.P, theta)

    def loss_and_grad(self, theta, t, want_grad=True, mu_fixed=None, head_range=None):
        return po.loss_and_grad(self.P, theta, t, want_grad, mu_fixed, head_range)

    def mean_field(self, theta):
        _, p_r, mu = po.cluster_stats(self.P, np.asarray(theta, dtype=np.float64))
        return po.mean_field(self.P, theta, p_r, mu)

    def epoch(self, theta, t):
        return po.epoch(self.P, theta, t)

    def philox(self, c, k):
        return po.philox4x32_10(c, k)


class CO(c_oracle.COracle):
    name = "c"

    def __init__(self, **kw):
        kw.pop("theta0", None)
        super().__init__(**kw)

    def mean_field(self, theta):
        _, _, A, B = self.loss_and_grad(theta, 0, want_grad=True, mean_field=True)
        return A, B


IMPLS = {"py": PyOracle, "c": CO}
