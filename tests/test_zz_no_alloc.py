"""The allocation-free form of the random-triplet count against the allocating one (same kernels, work space in the
library's code object instead of a buffer of the call): equal counts, call after call, also when a later call is
smaller than the one before it."""
import numpy as np
import pytest
import torch

from oracle import metrics_oracle as mo
from paper_2505_15511_amd import random_triplet_accuracy, random_triplet_accuracy_noalloc, workloads

pytestmark = pytest.mark.gpu


def _spaces(n, d, d_low, seed):
    X, _ = workloads.gmm_points(n, d, 8, 16.0, seed, mix="dirichlet", interleave=True)
    X = X.numpy()
    Y = (X[:, :d_low] + 0.5 * np.random.default_rng(seed).normal(size=(n, d_low))).astype(np.float32)
    return X, Y


def test_no_alloc_call_equals_the_allocating_call_twice_in_a_row():
    X, Y = _spaces(5000, 48, 2, 11)
    Xd, Yd = torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda()
    # first call: several launches (more than 2^24 triplets); second call: a smaller input and count, which must not
    # see anything the first left in the shared work space
    for (rows, T, seed) in ((5000, (1 << 24) + 70001, 5), (700, 30011, 6), (5000, 0, 7), (3, 1000, 8)):
        print(f"no-alloc triplets rows={rows} T={T} seed={seed}", flush=True)
        xs, ys = Xd[:rows].contiguous(), Yd[:rows].contiguous()
        before = torch.cuda.memory_allocated()
        got = random_triplet_accuracy_noalloc(xs, ys, T, seed)[0]
        assert torch.cuda.memory_allocated() == before
        assert got == random_triplet_accuracy(xs, ys, T, seed)[0]
        if T <= 100000:
            assert got == (mo.random_triplet_accuracy(X[:rows], Y[:rows], T, seed)[0] if T else 0)


def test_no_alloc_call_takes_device_memory_only():
    X, Y = _spaces(100, 8, 2, 1)
    with pytest.raises(ValueError):
        random_triplet_accuracy_noalloc(X, Y, 10, 0)
