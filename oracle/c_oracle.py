"""ctypes front end of the C oracle (oracle/nomad_oracle.c) -- TEST INFRASTRUCTURE, NOT PRODUCT.

Argument marshalling only; every number comes from the C file.  ``build()`` compiles it with
gcc (-O2, OpenMP) next to the source."""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nomad_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Problem(C.Structure):
    _fields_ = [("n", C.c_int64), ("row_ptr", C.c_void_p), ("col_idx", C.c_void_p), ("weights", C.c_void_p),
                ("cluster_of", C.c_void_p), ("n_clusters", C.c_int32), ("cluster_group", C.c_void_p),
                ("n_neg", C.c_int32), ("noise_count", C.c_double), ("seed", C.c_uint64),
                ("pool_size", C.c_int32), ("pool_block", C.c_int32), ("batches_per_epoch", C.c_int32),
                ("head_begin", C.c_int64), ("head_end", C.c_int64), ("sampled_far_field", C.c_int32),
                ("mean_gradient", C.c_int32), ("pool_mode", C.c_int32), ("pool_line", C.c_int32),
                ("pool_segment", C.c_int32)]


def _load():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_loss_grad.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]
        _lib.oracle_negatives.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_int64, C.c_void_p]
        _lib.oracle_cluster_stats.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        _lib.oracle_epoch.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_double, C.c_void_p, C.c_void_p]
        _lib.oracle_train.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_double, C.c_void_p]
        _lib.oracle_mean_field_at.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        _lib.oracle_philox4x32_10.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class COracle:
    """Holds int32/fp32 copies of a problem and calls the C oracle on them."""

    def __init__(self, *, n, row_ptr, col_idx, cluster_of, n_clusters, n_neg, noise_count, seed=0, n_epochs=1,
                 lr0=1.0, weights=None, cluster_group=None, pool_size=0, pool_block=0, batches_per_epoch=1,
                 sampled_far_field=False, mean_gradient=False, pool_mode=0, pool_line=1, pool_segment=64,
                 inverse_rank_weights=False, **_ignored):
        self.lib = _load()
        self.n = int(n)
        self.row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
        self.col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
        self.cluster_of = np.ascontiguousarray(cluster_of, dtype=np.int32)
        if inverse_rank_weights:                 # p(j|i) from the position of j in i's row (Eq. 7): the Python oracle's table
            from .nomad_oracle import rank_model_weights
            assert weights is None, "either explicit weights or the rank model"
            weights = rank_model_weights(self.row_ptr)
        self.weights = None if weights is None else np.ascontiguousarray(weights, dtype=np.float32)
        self.cluster_group = None if cluster_group is None else np.ascontiguousarray(cluster_group, dtype=np.int32)
        self.n_clusters = int(n_clusters)
        self.n_neg = int(n_neg)
        self.noise_count = float(noise_count) if noise_count > 0 else float(n_neg)
        self.seed = int(seed)
        self.n_epochs = int(n_epochs)
        self.lr0 = float(lr0)
        self.pool_size, self.pool_block = int(pool_size), int(pool_block)
        assert (self.pool_size == 0) == (self.pool_block == 0), "pool_size and pool_block go together"
        assert self.pool_size == 0 or self.cluster_group is None, "the pooled sampler needs a single population"
        self.P = _Problem(self.n, _ptr(self.row_ptr), _ptr(self.col_idx), _ptr(self.weights), _ptr(self.cluster_of),
                          self.n_clusters, _ptr(self.cluster_group), self.n_neg, self.noise_count, self.seed,
                          self.pool_size, self.pool_block, int(batches_per_epoch), 0, -1, int(bool(sampled_far_field)),
                          int(bool(mean_gradient)), int(pool_mode), int(pool_line), int(pool_segment))
        self.pool_mode, self.pool_line, self.pool_segment = int(pool_mode), int(pool_line), int(pool_segment)
        if self.pool_mode in (1, 2):
            Pz, ln = self.pool_size, self.pool_line
            assert 2 <= Pz <= 4096 and Pz & (Pz - 1) == 0, "distinct picks: the pool size is a power of two, 2..4096"
            assert ln >= 1 and ln & (ln - 1) == 0 and Pz % ln == 0 and self.n_neg <= Pz // ln, "lines: a power of two, s <= lines"
            sg = self.pool_segment
            assert sg >= 64 and sg & (sg - 1) == 0 and self.pool_block % sg == 0, "blocks are whole segments; segments a power of two >= 64"
            assert int(batches_per_epoch) == 1, "distinct picks: one step per epoch"
        else:
            assert self.pool_mode == 0 and self.pool_line == 1
        assert not (mean_gradient and (sampled_far_field or int(batches_per_epoch) > 1)), \
            "gradient through the means: exact far field, one step per epoch"
        assert not (sampled_far_field and self.pool_size), "sampled far field and pooled sampler do not combine"
        self.batches_per_epoch = int(batches_per_epoch)

    @property
    def n_edges(self):
        return int(self.row_ptr[-1])

    @property
    def threads(self):
        return int(self.lib.oracle_num_threads())

    def negatives(self, t, e_begin=0, e_end=None):
        e_end = self.n_edges if e_end is None else e_end
        out = np.zeros((e_end - e_begin, self.n_neg), dtype=np.int32)
        rc = self.lib.oracle_negatives(C.byref(self.P), t, e_begin, e_end, _ptr(out))
        assert rc == 0, rc
        return out

    def cluster_stats(self, theta):
        th = np.ascontiguousarray(theta, dtype=np.float32)
        counts = np.zeros(self.n_clusters, dtype=np.int64)
        mu = np.zeros((self.n_clusters, 2), dtype=np.float64)
        rc = self.lib.oracle_cluster_stats(C.byref(self.P), _ptr(th), _ptr(counts), _ptr(mu))
        assert rc == 0, rc
        return counts, counts / float(self.n), mu

    def loss_and_grad(self, theta, t, want_grad=True, mean_field=False, mu_fixed=None, head_range=None):
        """head_range = (begin, end): only the edges of those heads (one sub-step of a minibatch epoch)."""
        self.P.head_begin, self.P.head_end = (0, -1) if head_range is None else (int(head_range[0]), int(head_range[1]))
        try:
            return self._loss_and_grad(theta, t, want_grad, mean_field, mu_fixed)
        finally:
            self.P.head_begin, self.P.head_end = 0, -1

    def _loss_and_grad(self, theta, t, want_grad, mean_field, mu_fixed):
        th = np.ascontiguousarray(theta, dtype=np.float32)
        muf = None if mu_fixed is None else np.ascontiguousarray(mu_fixed, dtype=np.float64)
        loss = C.c_double(0.0)
        g = np.zeros((self.n, 2), dtype=np.float64) if want_grad else None
        A = np.zeros(self.n, dtype=np.float64) if mean_field else None
        B = np.zeros((self.n, 2), dtype=np.float64) if mean_field else None
        rc = self.lib.oracle_loss_grad(C.byref(self.P), _ptr(th), t, C.byref(loss), _ptr(g), None, 0, _ptr(A), _ptr(B), _ptr(muf))
        assert rc == 0, rc
        if mean_field:
            return loss.value, g, A, B
        return loss.value, g

    def grad_at(self, theta, t, points):
        """Gradient rows of the listed points only (single outputs computed one by one)."""
        th = np.ascontiguousarray(theta, dtype=np.float32)
        pts = np.asarray(points, dtype=np.int64)
        slot = np.full(self.n, -1, dtype=np.int32)
        slot[pts] = np.arange(len(pts), dtype=np.int32)
        g = np.zeros((len(pts), 2), dtype=np.float64)
        rc = self.lib.oracle_loss_grad(C.byref(self.P), _ptr(th), t, None, _ptr(g), _ptr(slot), len(pts), None, None, None)
        assert rc == 0, rc
        return g

    def mean_field_at(self, theta, heads):
        """A [m], B [m, 2] of the listed heads only, each from the loop over all cells."""
        th = np.ascontiguousarray(theta, dtype=np.float32)
        hd = np.ascontiguousarray(heads, dtype=np.int64)
        A = np.zeros(len(hd), dtype=np.float64)
        B = np.zeros((len(hd), 2), dtype=np.float64)
        rc = self.lib.oracle_mean_field_at(C.byref(self.P), _ptr(th), _ptr(hd), len(hd), _ptr(A), _ptr(B))
        assert rc == 0, rc
        return A, B

    def epoch(self, theta, t):
        th = np.array(theta, dtype=np.float32, copy=True, order="C")
        g = np.zeros((self.n, 2), dtype=np.float64)
        loss = C.c_double(0.0)
        rc = self.lib.oracle_epoch(C.byref(self.P), _ptr(th), t, self.n_epochs, self.lr0, _ptr(g), C.byref(loss))
        assert rc == 0, rc
        return th, g, loss.value

    def train(self, theta, t_begin=0, t_end=None):
        t_end = self.n_epochs if t_end is None else t_end
        th = np.array(theta, dtype=np.float32, copy=True, order="C")
        curve = np.zeros(max(0, t_end - t_begin), dtype=np.float64)
        rc = self.lib.oracle_train(C.byref(self.P), _ptr(th), t_begin, t_end, self.n_epochs, self.lr0, _ptr(curve))
        assert rc == 0, rc
        return th, curve

    def philox(self, counter, key):
        c = np.asarray(counter, dtype=np.uint32)
        k = np.asarray(key, dtype=np.uint32)
        out = np.zeros(4, dtype=np.uint32)
        self.lib.oracle_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
        return tuple(int(x) for x in out)


def philox(counter, key):
    lib = _load()
    c = np.asarray(counter, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib.oracle_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return tuple(int(x) for x in out)
