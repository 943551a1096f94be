#!/usr/bin/env python3
"""Writes tests/golden/oracle_tiny_case.txt: loss, gradient, negatives and one epoch of the Python oracle on a
fixed 12-point problem (grouped cells, weights, 3 negatives per edge), for the i.i.d. sampler, the pooled sampler
and a 3-batch epoch.  Calls only oracle/; run from the repository root:

    python tests/golden/make_oracle_golden.py

The file guards the oracle itself against silent changes: tests/test_oracle_golden.py recomputes every number
with both oracle implementations.  Regenerate it only together with a stated reason for the change in the
oracle's arithmetic."""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import nomad_oracle as po  # noqa: E402


def tiny_problem(**over):
    n = 12
    nbrs = {i: sorted({(i + 1) % n, (i + 5) % n, (i * 7 + 3) % n} - {i}) for i in range(n)}
    row_ptr = np.concatenate([[0], np.cumsum([len(nbrs[i]) for i in range(n)])])
    col = np.concatenate([nbrs[i] for i in range(n)])
    weights = (1.0 + (np.arange(len(col)) % 4) * 0.5).astype(np.float32)
    kw = dict(n=n, row_ptr=row_ptr, col_idx=col, cluster_of=np.arange(n) % 4, n_clusters=4, n_neg=3, noise_count=4.0,
              seed=(0xABCD << 32) | 0x1234, n_epochs=4, lr0=0.25, weights=weights, cluster_group=np.array([0, 1, 0, 1]))
    kw.update(over)
    return po.Problem(**kw)


def theta0():
    k = np.arange(12, dtype=np.float64)
    return np.stack([np.cos(0.9 * k) * (1 + 0.1 * k), np.sin(1.7 * k) * 0.8], 1).astype(np.float32)


def cases():
    yield "iid", tiny_problem()
    yield "pooled", tiny_problem(cluster_group=None, pool_size=5, pool_block=8)
    yield "batches3", tiny_problem(batches_per_epoch=3)


def main():
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_tiny_case.txt")
    with open(out, "w") as fh:
        fh.write("# written by tests/golden/make_oracle_golden.py from oracle/nomad_oracle.py (fp64, repr precision)\n")
        for name, P in cases():
            th = theta0()
            L, g = po.loss_and_grad(P, th, 2)
            th1, g_last, L_ep = po.epoch(P, th, 1)
            fh.write(f"case {name}\n")
            fh.write("negatives_t2 " + " ".join(str(int(x)) for x in po.negatives(P, 2).reshape(-1)) + "\n")
            fh.write(f"loss_t2 {float(L)!r}\n")
            fh.write("grad_t2 " + " ".join(repr(float(x)) for x in g.reshape(-1)) + "\n")
            fh.write(f"epoch1_loss {float(L_ep)!r}\n")
            fh.write("epoch1_theta " + " ".join(repr(float(x)) for x in th1.reshape(-1)) + "\n")
    print("wrote", out)


if __name__ == "__main__":
    main()
