"""Host logic of bench.py that needs no GPU: the byte model of the roofline, the committed counter figures it reads and the
check that says whether they still describe the kernel that was timed, and the refusal of more than one GPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_algorithmic_bytes_of_the_benchmark_edge_pass():
    # configuration 4: 96 B per directed edge (col 4, theta_j 8, the tail's coefficient 4, s = 5 rows read and forces
    # handed on 80) and 20 B per point (row_ptr 4, theta_i 8, head gradient 8)
    E, n = 299_112_914, 10_000_000
    assert bench.algorithmic_bytes("edges", n, E, 5, 4096, False, False, True) == 96 * E + 20 * n
    # atomic mode accumulates the tail's force (8 B) instead of handing on a coefficient (4 B)
    assert bench.algorithmic_bytes("edges", n, E, 5, 4096, False, False, False) == 100 * E + 20 * n
    # pooled samplers: rows and forces once per pool entry and block
    blocks = (E + 8191) // 8192
    assert bench.algorithmic_bytes("edges", n, E, 5, 4096, False, False, True, (2048, 8192)) == 16 * E + 16 * 2048 * blocks + 20 * n


WORKLOADS = [(cfg, "det", "iid", k) for cfg in (1, 2, 3, 4, 5) for k in ("edges", "tiles")] + \
            [(5, "det", "iid", "mean_field"), (4, "atomic", "iid", "edges")] + \
            [(4, "det", smp, k) for smp in ("pooled_exact", "pooled_stratified") for k in ("edges", "tiles")]


@pytest.mark.parametrize("cfg,mode,sampler,kernel", WORKLOADS)
def test_every_timed_kernel_has_counter_figures(cfg, mode, sampler, kernel):
    traffic, ms = bench.measured_traffic(kernel, cfg, mode, 1.0, sampler)
    assert traffic is not None and traffic > 0
    assert ms is not None and ms > 0
    # per launch: an epoch cut into four launches moves a quarter each
    assert bench.measured_traffic(kernel, cfg, mode, 4.0, sampler)[0] == pytest.approx(traffic / 4)


def test_traffic_is_flagged_when_the_kernel_has_changed():
    _, ms = bench.measured_traffic("edges", 4, "det")
    same = {"kernel": "edges", "launches_per_epoch": 4.0}
    bench.attach_traffic(same, ms * 1.04, 4, "det")
    assert same["traffic_current"] is True and same["traffic_counted_at_ms_per_epoch"] == ms
    faster = {"kernel": "edges", "launches_per_epoch": 4.0}
    bench.attach_traffic(faster, ms * 0.7, 4, "det")
    assert faster["traffic_current"] is False and faster["traffic"] == same["traffic"]
    unknown = {"kernel": "edges"}
    bench.attach_traffic(unknown, 1.0, 4, "det", "no such sampler")
    assert unknown["traffic"] is None and "traffic_current" not in unknown


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
