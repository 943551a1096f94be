"""The C oracle built with AddressSanitizer and UndefinedBehaviorSanitizer (gcc, host only) and run over every entry
point on the kinds of problems the pins use; the sums it prints must be those of the ordinary build."""
import ctypes as C
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import c_oracle
from paper_2505_15511_amd.workloads import random_symmetric_graph

ORACLE_DIR = os.path.dirname(os.path.abspath(c_oracle.__file__))


@pytest.fixture(scope="module")
def sanitized(tmp_path_factory):
    if not shutil.which("gcc"):
        pytest.skip("no C compiler")
    exe = tmp_path_factory.mktemp("san") / "sanitize_check"
    subprocess.run(["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
                    "-Wall", "-Werror", os.path.join(ORACLE_DIR, "nomad_oracle.c"), os.path.join(ORACLE_DIR, "sanitize_check.c"),
                    "-o", str(exe), "-lm"], check=True)
    return str(exe)


def _weighted(v):
    v = np.asarray(v, dtype=np.float64).reshape(-1)
    return float((v * (np.arange(len(v)) % 97 + 1)).sum())


CASES = {
    "plain": dict(groups=False, weights=False),
    "grouped-weighted": dict(groups=True, weights=True),
    "sub-steps": dict(groups=True, weights=True, batches_per_epoch=3),
    "sampled-far-field": dict(groups=True, weights=False, sampled_far_field=True),
    "mean-gradient": dict(groups=True, weights=True, mean_gradient=True),
    "pooled-16-bit-picks": dict(groups=False, weights=True, pool_size=12, pool_block=40),
    "pooled-distinct-picks": dict(groups=False, weights=False, pool_size=16, pool_block=128, pool_mode=1, pool_line=2, pool_segment=64),
    "no-negatives": dict(groups=True, weights=False, s=0),
    "idle-points-and-empty-cluster": dict(groups=True, weights=False, idle=True),
}


@pytest.mark.parametrize("case", list(CASES))
def test_sanitized_oracle_runs_clean_and_agrees_with_the_ordinary_build(sanitized, case, tmp_path):
    opt = dict(CASES[case])
    n, R = 70, 6
    s = opt.pop("s", 3)
    rng = np.random.default_rng(len(case))
    row_ptr, col = random_symmetric_graph(n - 4 if opt.get("idle") else n, 5.0, 7)
    if opt.pop("idle", False):                                    # four points without edges; cluster 5 stays empty
        row_ptr = np.concatenate([row_ptr, np.full(4, row_ptr[-1])])
        cluster = rng.integers(0, R - 1, n)
    else:
        cluster = rng.integers(0, R, n)
        cluster[:R] = np.arange(R)
    E = len(col)
    kw = dict(n=n, row_ptr=row_ptr.astype(np.int32), col_idx=col.astype(np.int32), cluster_of=cluster.astype(np.int32), n_clusters=R,
              n_neg=s, noise_count=4.0, seed=0x1234567890, n_epochs=4, lr0=0.3)
    if opt.pop("weights"):
        kw["weights"] = rng.uniform(0.2, 2.0, E).astype(np.float32)
    if opt.pop("groups"):
        kw["cluster_group"] = (np.arange(R) % 3).astype(np.int32)
    kw.update(opt)
    theta = (rng.normal(size=(n, 2)) * 0.8).astype(np.float32)
    kw["row_ptr"].tofile(tmp_path / "row_ptr.i32")
    kw["col_idx"].tofile(tmp_path / "col.i32")
    kw["cluster_of"].tofile(tmp_path / "cluster.i32")
    theta.tofile(tmp_path / "theta.f32")
    if "weights" in kw:
        kw["weights"].tofile(tmp_path / "weights.f32")
    if "cluster_group" in kw:
        kw["cluster_group"].tofile(tmp_path / "group.i32")
    args = [sanitized, str(tmp_path), n, E, R, s, 4.0, kw.get("pool_size", 0), kw.get("pool_block", 0), kw.get("pool_mode", 0),
            kw.get("pool_line", 1), kw.get("pool_segment", 64), kw.get("batches_per_epoch", 1), int(kw.get("sampled_far_field", False)),
            int(kw.get("mean_gradient", False))]
    run = subprocess.run([str(a) for a in args], capture_output=True, text=True, env={**os.environ, "OMP_NUM_THREADS": "3"})
    assert run.returncode == 0, run.stdout + run.stderr                 # a sanitizer report ends the program with an error
    got = {line.split()[0]: [float(x) for x in line.split()[1:]] for line in run.stdout.splitlines()}

    O = c_oracle.COracle(**kw)
    neg = O.negatives(3).astype(np.int64).reshape(-1)
    assert got["negatives"][0] == float((neg * (np.arange(len(neg)) % 31 + 1)).sum())
    L, g, A, B = O.loss_and_grad(theta, 3, mean_field=True)
    close = lambda a, b: abs(a - b) <= 1e-11 * max(1.0, abs(b))           # the thread count differs: sums in another order
    assert close(got["loss"][0], L) and close(got["grad"][0], _weighted(g)) and close(got["A"][0], _weighted(A)) and close(got["B"][0], _weighted(B))
    pts = np.array([n - 1, 0, n // 2])
    if not kw.get("mean_gradient"):
        assert np.allclose(got["rows"], O.grad_at(theta, 3, pts).reshape(-1), rtol=0, atol=1e-12)
    hA, hB = O.mean_field_at(theta, pts)
    assert close(got["mean_field_at"][0], hA[0] + 2 * hA[1] + 3 * hA[2]) and close(got["mean_field_at"][1], _weighted(hB))
    th1, _, eloss = O.epoch(theta, 1)
    assert close(got["epoch"][0], eloss) and close(got["epoch"][1], _weighted(th1))
    th4, curve = O.train(th1, 1, 4)
    assert close(got["train"][0], curve[2]) and close(got["train"][1], _weighted(th4))
