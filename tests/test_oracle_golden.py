"""The oracle against its own frozen outputs (tests/golden/oracle_tiny_case.txt, written by
tests/golden/make_oracle_golden.py, which calls only oracle/): guards both implementations against silent changes."""
import importlib.util
import os

import numpy as np
import pytest

from oracle import c_oracle, nomad_oracle as po

HERE = os.path.dirname(os.path.abspath(__file__))
_spec = importlib.util.spec_from_file_location("make_oracle_golden", os.path.join(HERE, "golden", "make_oracle_golden.py"))
gold = importlib.util.module_from_spec(_spec)
_spec.loader.exec_module(gold)


def _read():
    cases, cur = {}, None
    for line in open(os.path.join(HERE, "golden", "oracle_tiny_case.txt")):
        if line.startswith("#"):
            continue
        key, _, rest = line.strip().partition(" ")
        if key == "case":
            cur = cases.setdefault(rest, {})
        else:
            cur[key] = rest.split()
    return cases


GOLD = _read()


@pytest.mark.parametrize("name", ["iid", "pooled", "batches3"])
def test_python_and_c_oracle_reproduce_the_frozen_case(name):
    P = dict(gold.cases())[name]
    want = GOLD[name]
    th = gold.theta0()
    kw = dict(n=P.n, row_ptr=P.row_ptr, col_idx=P.col_idx, cluster_of=P.cluster_of, n_clusters=P.n_clusters, n_neg=P.n_neg,
              noise_count=P.noise_count, seed=P.seed, n_epochs=P.n_epochs, lr0=P.lr0, weights=P.weights,
              cluster_group=P.cluster_group, pool_size=P.pool_size, pool_block=P.pool_block,
              batches_per_epoch=P.batches_per_epoch)
    C = c_oracle.COracle(**kw)
    neg = np.array(want["negatives_t2"], dtype=np.int64).reshape(-1, P.n_neg)
    assert np.array_equal(po.negatives(P, 2), neg) and np.array_equal(C.negatives(2), neg)
    L_want, g_want = float(want["loss_t2"][0]), np.array(want["grad_t2"], dtype=np.float64).reshape(-1, 2)
    for L, g in (po.loss_and_grad(P, th, 2), C.loss_and_grad(th, 2)):
        assert abs(L - L_want) < 1e-13 and np.abs(g - g_want).max() < 1e-13
    th_want = np.array(want["epoch1_theta"], dtype=np.float64).reshape(-1, 2)
    for th1, _, L_ep in (po.epoch(P, th, 1), C.epoch(th, 1)):
        assert np.abs(th1.astype(np.float64) - th_want).max() < 1e-6 and abs(L_ep - float(want["epoch1_loss"][0])) < 1e-12
