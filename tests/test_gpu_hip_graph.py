"""nomad_epoch only enqueues kernels on the caller's stream, so a caller can record a run of epochs into a HIP graph
and replay it: the launch-bound small configurations then pay one graph launch instead of two kernel launches per
epoch.  Replays are checked against the eager run, several times, with eager work in between."""
import numpy as np
import pytest
import torch

from paper_2505_15511_amd import Nomad, SCATTER_ATOMIC, SCATTER_DETERMINISTIC, workloads

pytestmark = pytest.mark.gpu


def _case(name):
    if name == "config1":
        return workloads.make_config(1)
    if name == "config3@0.02-groups":
        return workloads.make_config(3, scale=0.02, n_groups=4)
    w = workloads.make_config(3, scale=0.02)
    w.pool_size, w.pool_block = 512, 2048
    return w


@pytest.mark.parametrize("case", ["config1", "config3@0.02-groups", "config3@0.02-pooled"])
def test_recorded_epochs_replay_like_the_eager_run(case):
    w = _case(case)
    T = 12
    theta0 = w.theta0.cuda()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        nm = Nomad.from_workload(w, SCATTER_DETERMINISTIC, stream=side.cuda_stream)
        for t in range(T):                       # eager run
            nm.epoch(t)
        side.synchronize()
        th_eager, g_eager = nm.get_embedding(), nm.get_gradient()
        nm.set_embedding(theta0)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for t in range(T):
                nm.epoch(t)
        for replay in range(3):
            nm.set_embedding(theta0)             # eager work between the replays
            if replay == 1:
                nm.epoch(0)
                nm.loss(3)
                nm.set_embedding(theta0)
            graph.replay()
            side.synchronize()
            assert np.array_equal(nm.get_embedding(), th_eager), replay
            assert np.array_equal(nm.get_gradient(), g_eager), replay
        nm.close()


def test_recorded_epochs_in_atomic_mode_stay_within_the_bar():
    w = workloads.make_config(1)
    T = 8
    theta0 = w.theta0.cuda()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        ref = Nomad.from_workload(w, SCATTER_DETERMINISTIC, stream=side.cuda_stream)
        nm = Nomad.from_workload(w, SCATTER_ATOMIC, stream=side.cuda_stream)
        for t in range(T):
            ref.epoch(t)
        nm.epoch(0)
        nm.set_embedding(theta0)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for t in range(T):
                nm.epoch(t)
        for _ in range(2):
            nm.set_embedding(theta0)
            graph.replay()
            side.synchronize()
            assert np.abs(nm.get_embedding() - ref.get_embedding()).max() < 1e-4
        nm.close()
        ref.close()
