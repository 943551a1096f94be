"""HIP path vs CPU oracle, element by element, through the C ABI (needs an MI355X)."""
import ctypes as C
import math

import numpy as np
import pytest
import torch

from oracle import c_oracle
from paper_2505_15511_amd import (Nomad, NomadError, PATH_ATOMIC_FP32, PATH_BINNED, PATH_BINNED_POOLED, PATH_FIXED_ATOMICS,
                                  SCATTER_ATOMIC, SCATTER_DETERMINISTIC, workloads)

pytestmark = pytest.mark.gpu

MODES = [pytest.param(SCATTER_DETERMINISTIC, id="det"), pytest.param(SCATTER_ATOMIC, id="atomic")]
GRAD_TOL = 1e-5   # max_i |g_i - g^_i|_inf / max_i |g^_i|_inf, the bar named for the deterministic path
LOSS_TOL = 1e-5   # relative


def grad_err(g, ref):
    return np.abs(np.asarray(g, dtype=np.float64) - ref).max() / np.abs(ref).max()


def grad_err_per_component(g, ref):
    """max over points and components of |g - ref| / max(|ref|, 1e-3 max|ref|): an error confined to points with small
    forces (tails of hubs, heads without edges, negatives that stood for a cell mean) shows here and not in
    grad_err.  Components near force balance are differences of float32 terms a hundred times their size, hence
    the looser bound."""
    ref = np.asarray(ref, dtype=np.float64)
    return (np.abs(np.asarray(g, dtype=np.float64) - ref) / np.maximum(np.abs(ref), 1e-3 * np.abs(ref).max())).max()


COMPONENT_TOL = 1e-3


def note(msg):
    print(msg, flush=True)


_cache = {}


def workload(cfg, scale=1.0, **kw):
    key = (cfg, scale, tuple(sorted(kw.items())))
    if key not in _cache:
        _cache[key] = workloads.make_config(cfg, scale=scale, **kw)
    return _cache[key]


def small_random(seed, n=3000, R=12, groups=True, weights=True, contiguous=False, s=3, M=4.0, T=20):
    """Random symmetric graph with interleaved (non-contiguous) clusters, weights and groups."""
    rng = np.random.default_rng(seed)
    g = workloads.planted_knn_graph(n, R, 6, 0.05, seed)
    cluster_of = g["cluster_of"].numpy().copy()
    row_ptr, col = g["row_ptr"].numpy(), g["col_idx"].numpy()
    if not contiguous:
        cluster_of = rng.permutation(cluster_of)
    w = rng.uniform(0.2, 2.0, len(col)).astype(np.float32) if weights else None
    grp = None
    if groups:
        grp = rng.integers(0, 4, R).astype(np.int32)
        grp[:4] = [0, 1, 2, 3]
    theta0 = (rng.normal(size=(n, 2)) * 0.5).astype(np.float32)
    return dict(n=n, row_ptr=row_ptr, col_idx=col, weights=w, cluster_of=cluster_of.astype(np.int32), n_clusters=R,
                cluster_group=grp, theta0=theta0, n_neg=s, noise_count=M, n_epochs=T, lr0=0.5, seed=seed * 31 + 7)


def make_nomad(d, mode, tune=None):
    nm = Nomad(d["n"], d["n_clusters"], d["n_neg"], d["noise_count"], d["n_epochs"], d["lr0"], d["seed"], mode,
               pool_size=d.get("pool_size", 0), pool_block=d.get("pool_block", 0),
               batches_per_epoch=d.get("batches_per_epoch", 1), sampled_far_field=d.get("sampled_far_field", False),
               mean_gradient=d.get("mean_gradient", False), pool_mode=d.get("pool_mode", 0), pool_line=d.get("pool_line", 0),
               pool_segment=d.get("pool_segment", 0), inverse_rank_weights=d.get("inverse_rank_weights", False), tune=tune)
    nm.set_graph(d["row_ptr"], d["col_idx"], None if d.get("inverse_rank_weights") else d["weights"], d["cluster_of"], d["cluster_group"])
    nm.set_embedding(d["theta0"])
    return nm


# ------------------------------------------------------------------ negatives: bit exact
@pytest.mark.parametrize("case", ["config1", "config3@0.05", "config5@1e-3", "random-groups"])
def test_negatives_bit_exact(case):
    note(f"negatives {case}")
    if case == "random-groups":
        d = small_random(3)
    else:
        cfg, _, sc = case.partition("@")
        d = workload(int(cfg[-1]), float(sc) if sc else 1.0).numpy()
    O = c_oracle.COracle(**d)
    with make_nomad(d, SCATTER_ATOMIC) as nm:
        assert nm.num_edges() == O.n_edges
        for t in (0, 7):
            assert np.array_equal(nm.get_negatives(t), O.negatives(t))
        E = O.n_edges
        assert np.array_equal(nm.get_negatives(3, E // 3, E // 3 + 1000), O.negatives(3, E // 3, E // 3 + 1000))
        assert nm.get_negatives(3, 5, 5).shape == (0, d["n_neg"])


# ------------------------------------------------------------------ cluster statistics
@pytest.mark.parametrize("case", ["config1", "config3@0.05", "random-groups"])
def test_cluster_counts_exact_and_means_close(case):
    note(f"means {case}")
    d = small_random(4) if case == "random-groups" else workload(int(case[6]), float(case.partition("@")[2] or 1)).numpy()
    rng = np.random.default_rng(1)
    theta = (rng.normal(size=(d["n"], 2)) * 3 + [10.0, -4.0]).astype(np.float32)
    O = c_oracle.COracle(**d)
    counts, _, mu = O.cluster_stats(theta)
    with make_nomad(d, SCATTER_ATOMIC) as nm:
        nm.set_embedding(theta)
        gmu, gcounts = nm.get_means()
        assert np.array_equal(gcounts, counts)
        assert np.abs(gmu - mu).max() < 1e-6 * max(1.0, np.abs(mu).max())
        # set/get round trip is the identity
        assert np.array_equal(nm.get_embedding(), theta)


def test_mean_field_sums():
    for d in (small_random(5), workload(5, 1e-3).numpy()):
        note(f"mean field n={d['n']}")
        O = c_oracle.COracle(**d)
        rng = np.random.default_rng(2)
        theta = (rng.normal(size=(d["n"], 2)) * 2).astype(np.float32)
        _, _, A, B = O.loss_and_grad(theta, 0, mean_field=True)
        with make_nomad(d, SCATTER_DETERMINISTIC) as nm:
            nm.set_embedding(theta)
            gA, gB = nm.get_mean_field()
        assert np.abs(gA - A).max() < 2e-6 * np.abs(A).max()
        assert np.abs(gB - B).max() < 2e-6 * np.abs(B).max()


# ------------------------------------------------------------------ gradient and loss
CASES = ["config1", "config2@0.1", "config3@0.05", "config5@1e-3", "random-groups", "random-plain", "random-contig"]


def _case(case):
    if case == "random-groups":
        return small_random(6)
    if case == "random-plain":
        return small_random(7, groups=False, weights=False, s=5, M=5.0)
    if case == "random-contig":
        return small_random(8, contiguous=True)
    cfg, _, sc = case.partition("@")
    return workload(int(cfg[-1]), float(sc) if sc else 1.0).numpy()


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("case", CASES)
def test_gradient_and_loss_after_one_epoch(case, mode):
    note(f"gradient {case} mode={mode}")
    d = _case(case)
    O = c_oracle.COracle(**d)
    th1, g_ref, _ = O.epoch(d["theta0"], 0)
    L_ref, _ = O.loss_and_grad(th1, 1, want_grad=False)
    with make_nomad(d, mode) as nm:
        nm.epoch(0)
        g = nm.get_gradient()
        err, err_c = grad_err(g, g_ref), grad_err_per_component(g, g_ref)
        L = nm.loss(1)
        th = nm.get_embedding()
    note(f"  grad err {err:.2e} (per component, floor 1e-3: {err_c:.2e})  loss {L:.8f} vs {L_ref:.8f}")
    assert err < GRAD_TOL and err_c < COMPONENT_TOL
    assert abs(L - L_ref) < LOSS_TOL * abs(L_ref)
    assert np.abs(th - th1).max() < 1e-5 * max(1.0, np.abs(th1).max())


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("case", ["config1", "config3@0.05", "random-groups"])
def test_mid_run_gradient_restarted_from_the_gpu_embedding(case, mode):
    """Run some epochs on the GPU, then hand its embedding to the oracle and compare the next gradient."""
    note(f"mid-run {case} mode={mode}")
    d = _case(case)
    O = c_oracle.COracle(**d)
    t_mid = min(10, d["n_epochs"] - 2)
    with make_nomad(d, mode) as nm:
        for t in range(t_mid):
            nm.epoch(t)
        theta = nm.get_embedding()
        nm.epoch(t_mid)
        g = nm.get_gradient()
    _, g_ref = O.loss_and_grad(theta, t_mid)
    err = grad_err(g, g_ref)
    note(f"  grad err {err:.2e}")
    assert err < GRAD_TOL
    assert np.abs(theta).max() > 0.05      # the embedding has actually moved away from the init


# ------------------------------------------------------------------ the two scatter paths
def test_deterministic_path_is_bit_reproducible_and_atomic_path_agrees():
    d = workload(3, 0.05).numpy()
    runs = []
    for mode in (SCATTER_DETERMINISTIC, SCATTER_DETERMINISTIC, SCATTER_ATOMIC):
        with make_nomad(d, mode) as nm:
            for t in range(5):
                nm.epoch(t)
            runs.append((nm.get_gradient(), nm.get_embedding()))
    assert np.array_equal(runs[0][0], runs[1][0]) and np.array_equal(runs[0][1], runs[1][1])
    scale = np.abs(runs[0][0]).max()
    assert np.abs(runs[0][0] - runs[2][0]).max() < 2e-5 * scale      # different summation order only
    assert np.abs(runs[0][1] - runs[2][1]).max() < 1e-4


def test_resume_from_embedding_and_epoch_index_is_bit_exact():
    d = workload(1).numpy()
    with make_nomad(d, SCATTER_DETERMINISTIC) as nm:
        for t in range(10):
            nm.epoch(t)
        straight = nm.get_embedding()
    with make_nomad(d, SCATTER_DETERMINISTIC) as nm:
        for t in range(5):
            nm.epoch(t)
        half = nm.get_embedding()
    with make_nomad(d, SCATTER_DETERMINISTIC) as nm:
        nm.set_embedding(half)
        for t in range(5, 10):
            nm.epoch(t)
        assert np.array_equal(nm.get_embedding(), straight)


# ------------------------------------------------------------------ the binned deterministic path
def skewed_degree_graph(seed, n=6000, hubs=3):
    """Directed graph whose rows range from one edge to several thousand: rows that end inside a wavefront,
    rows that straddle wavefronts, and hub rows that span several rounds and workgroups of the edge pass."""
    rng = np.random.default_rng(seed)
    deg = rng.integers(1, 40, n)
    deg[rng.choice(n, 40, replace=False)] = rng.integers(65, 300, 40)
    deg[rng.choice(n, hubs, replace=False)] = rng.integers(1500, 4000, hubs)
    deg[rng.choice(n, 50, replace=False)] = 0
    rows, cols = [], []
    for i in range(n):
        c = rng.choice(n - 1, int(deg[i]), replace=False)
        c[c >= i] += 1                               # no self loops, distinct tails
        cols.append(np.sort(c))
    row_ptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    R = 7
    return dict(n=n, row_ptr=row_ptr, col_idx=np.concatenate(cols).astype(np.int32), weights=None,
                cluster_of=rng.integers(0, R, n).astype(np.int32), n_clusters=R, cluster_group=None,
                theta0=(rng.normal(size=(n, 2)) * 0.7).astype(np.float32), n_neg=5, noise_count=5.0, n_epochs=10, lr0=0.2,
                seed=seed + 99)


@pytest.mark.parametrize("tune,path", [({}, PATH_BINNED), ({"edge_block": 512}, PATH_BINNED), ({"workgroups_per_cu": 3}, PATH_BINNED),
                                       ({"scatter_path": PATH_FIXED_ATOMICS}, PATH_FIXED_ATOMICS), ({"record_phases": 3}, PATH_BINNED),
                                       ({"record_sort": 2}, PATH_BINNED), ({"record_sort": 2, "edge_block": 512, "record_phases": 3}, PATH_BINNED)],
                         ids=["1024-lane", "512-lane", "3-per-cu", "fixed-point-atomics", "3-phases", "unsorted-records",
                              "unsorted-512-lane-3-phases"])
def test_deterministic_variants_on_skewed_degrees(tune, path):
    """Every launch shape of the deterministic path gives the oracle's gradient, and the same embedding bit for bit
    when run twice, on rows of very different lengths; the library says which path it runs."""
    env = tune
    d = skewed_degree_graph(4)
    O = c_oracle.COracle(**d)
    th1, g_ref, _ = O.epoch(d["theta0"], 0)
    out = []
    for _ in range(2):
        with make_nomad(d, SCATTER_DETERMINISTIC, tune=tune) as nm:
            assert nm.scatter_path() == path and (nm.note() == "") == (path == PATH_BINNED) and nm.device_bytes() > 0
            nm.epoch(0)
            g = nm.get_gradient()
            nm.epoch(1)
            out.append((g, nm.get_embedding()))
    note(f"  {env}: grad err {grad_err(out[0][0], g_ref):.2e} (per component, floor 1e-3: {grad_err_per_component(out[0][0], g_ref):.2e})")
    assert grad_err(out[0][0], g_ref) < GRAD_TOL and grad_err_per_component(out[0][0], g_ref) < COMPONENT_TOL
    assert np.array_equal(out[0][0], out[1][0]) and np.array_equal(out[0][1], out[1][1])


@pytest.mark.parametrize("case", ["skewed", "config5@0.001", "config3@0.05", "config5@0.001-3-sub-steps", "config3@0.05-pooled-general-kernels"])
def test_sorted_and_unsorted_records_give_the_same_bits(case):
    """A round's records written after a counting sort by tile, or by the lanes that made them: the tile sums are integer
    sums of the same records, so gradient and embedding agree bit for bit (and with the library's own choice)."""
    d = skewed_degree_graph(5) if case == "skewed" else dict(workload(int(case[6]), float(case.split("@")[1].split("-")[0])).numpy())
    if case.endswith("sub-steps"):
        d["batches_per_epoch"] = 3
    if case.endswith("general-kernels"):
        d["pool_size"], d["pool_block"] = 48, 100      # a block that is no multiple of 1024: the general kernels draw from the pools
    runs = []
    for tune in ({}, {"record_sort": 1}, {"record_sort": 2}, {"record_sort": 2, "flush_rounds": 1}):
        with make_nomad(d, SCATTER_DETERMINISTIC, tune=tune) as nm:
            assert nm.scatter_path() == PATH_BINNED
            for t in range(3):
                nm.epoch(t)
            runs.append((nm.get_gradient(), nm.get_embedding()))
    for g, th in runs[1:]:
        assert np.array_equal(g, runs[0][0]) and np.array_equal(th, runs[0][1])
    O = c_oracle.COracle(**d)
    _, g_ref, _ = O.epoch(d["theta0"], 0)
    with make_nomad(d, SCATTER_DETERMINISTIC, tune={"record_sort": 2}) as nm:
        nm.epoch(0)
        g = nm.get_gradient()
    note(f"  {case}, unsorted records: grad err {grad_err(g, g_ref):.2e} (per component: {grad_err_per_component(g, g_ref):.2e})")
    assert grad_err(g, g_ref) < GRAD_TOL and grad_err_per_component(g, g_ref) < COMPONENT_TOL


def test_record_phases_change_the_pool_size_and_nothing_else():
    """The edge pass of a step in 1, 3, 8 or 64 phases (sums carried from phase to phase in 64-bit fixed point): gradient
    and embedding are the same bit for bit, the library holds less memory, and the knob is refused once the graph is set."""
    d = dict(workload(3, 0.05).numpy())
    runs = []
    for phases in (1, 3, 8, 64):
        for sub_steps in (1, 3):
            with make_nomad(dict(d, batches_per_epoch=sub_steps), SCATTER_DETERMINISTIC, tune={"record_phases": phases}) as nm:
                assert nm.scatter_path() == PATH_BINNED
                for t in range(3):
                    nm.epoch(t)
                runs.append((phases, sub_steps, nm.get_gradient(), nm.get_embedding(), nm.device_bytes()))
                with pytest.raises(NomadError, match="ORDER"):
                    nm._check(nm.lib.nomad_tune(nm.ctx, 5, 2))
    for sub_steps in (1, 3):
        same = [r for r in runs if r[1] == sub_steps]
        for r in same[1:]:
            assert np.array_equal(r[2], same[0][2]) and np.array_equal(r[3], same[0][3]), (r[0], sub_steps)
        assert same[2][4] < same[0][4]                    # eight phases hold a smaller pool than one
    _, g_ref, _ = c_oracle.COracle(**d).epoch(runs[0][3] * 0 + d["theta0"], 0)   # and they are the oracle's numbers
    with make_nomad(d, SCATTER_DETERMINISTIC, tune={"record_phases": 8}) as nm:
        nm.epoch(0)
        assert grad_err(nm.get_gradient(), g_ref) < GRAD_TOL


# ------------------------------------------------------------------ the opt-in pooled sampler
POOLS = [pytest.param((48, 100), id="P48-G100-general-kernels"), pytest.param((2048, 4096), id="P2048-G4096"),
         pytest.param((1000, 1024), id="P1000-G1024"), pytest.param((4096, 2048), id="P4096-G2048"),
         pytest.param((512, 8192), id="P512-G8192")]


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("pool", POOLS)
def test_pooled_sampler_negatives_gradient_and_loss(pool, mode):
    for case in ("config3@0.05", "skewed"):
        d = dict(workload(3, 0.05).numpy()) if case != "skewed" else skewed_degree_graph(6)
        d["pool_size"], d["pool_block"] = pool
        O = c_oracle.COracle(**d)
        th1, g_ref, _ = O.epoch(d["theta0"], 0)
        L_ref, _ = O.loss_and_grad(th1, 1, want_grad=False)
        with make_nomad(d, mode) as nm:
            assert np.array_equal(nm.get_negatives(0), O.negatives(0))
            assert np.array_equal(nm.get_negatives(3, 1000, 9000), O.negatives(3, 1000, 9000))
            nm.epoch(0)
            err = grad_err(nm.get_gradient(), g_ref)
            L = nm.loss(1)
        note(f"  pooled {pool} {case} mode={mode}: grad err {err:.2e}  loss {L:.8f} vs {L_ref:.8f}")
        assert err < GRAD_TOL
        assert abs(L - L_ref) < LOSS_TOL * abs(L_ref)


# pool size, block, points per line, segment: the fast kernel at 1, 2, 4 and 8 rounds, lines of 1 to 64 points, blocks of
# consecutive positions (segment = block) and spread blocks, and shapes only the general kernels take
DISTINCT = [pytest.param((2048, 4096, 16, 256), id="P2048-G4096-line16-seg256"), pytest.param((4096, 8192, 16, 64), id="P4096-G8192-line16-seg64"),
            pytest.param((1024, 1024, 1, 1024), id="P1024-G1024-line1-consecutive"), pytest.param((512, 2048, 64, 1024), id="P512-G2048-line64-seg1024"),
            pytest.param((64, 8192, 4, 8192), id="P64-G8192-line4-consecutive"), pytest.param((16, 192, 2, 64), id="P16-G192-general-kernels"),
            pytest.param((256, 4096, 8, 2048), id="P256-G4096-line8-seg2048")]


# the same sampler with stratified pools (pool_mode 2): the last field
STRATIFIED = [pytest.param((2048, 8192, 16, 256, 2), id="stratified-P2048-G8192-line16-seg256"),
              pytest.param((1024, 1024, 1, 64, 2), id="stratified-P1024-G1024-line1-seg64"),
              pytest.param((4096, 4096, 64, 4096, 2), id="stratified-P4096-G4096-line64-consecutive"),
              pytest.param((4096, 2048, 1, 256, 2), id="stratified-P4096-G2048-line1-seg256"),      # more lines than lanes
              pytest.param((2048, 8192, 1, 256, 2), id="stratified-P2048-G8192-line1-seg256"),
              pytest.param((32, 320, 4, 64, 2), id="stratified-P32-G320-general-kernels")]


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("pool", DISTINCT + STRATIFIED)
def test_pooled_sampler_with_distinct_picks_negatives_gradient_and_loss(pool, mode):
    pool_mode = pool[4] if len(pool) == 5 else 1
    pool = pool[:4]
    for case in ("config3@0.05", "skewed", "tiny"):
        d = dict(workload(3, 0.05).numpy()) if case == "config3@0.05" else skewed_degree_graph(6) if case == "skewed" else \
            small_random(9, n=300, groups=False, weights=True, s=5, M=5.0)
        d["pool_size"], d["pool_block"], d["pool_line"], d["pool_segment"] = pool
        d["pool_mode"] = pool_mode
        O = c_oracle.COracle(**d)
        E = len(d["col_idx"])
        th1, g_ref, _ = O.epoch(d["theta0"], 0)
        L_ref, _ = O.loss_and_grad(th1, 1, want_grad=False)
        with make_nomad(d, mode) as nm:
            if mode == SCATTER_DETERMINISTIC:
                assert nm.scatter_path() == (PATH_BINNED_POOLED if pool[1] % 1024 == 0 else PATH_BINNED)
            assert np.array_equal(nm.get_negatives(0), O.negatives(0))
            assert np.array_equal(nm.get_negatives(3, E // 7, E // 7 + min(E // 2, 8000)), O.negatives(3, E // 7, E // 7 + min(E // 2, 8000)))
            nm.epoch(0)
            g = nm.get_gradient()
            err, err_c = grad_err(g, g_ref), grad_err_per_component(g, g_ref)
            L = nm.loss(1)
            th = nm.get_embedding()
            th2_ref, g2_ref, _ = O.epoch(th, 1)            # a second epoch from the library's own embedding
            nm.epoch(1)
            err2 = grad_err(nm.get_gradient(), g2_ref)
        note(f"  distinct picks {pool} {case} mode={mode}: grad err {err:.2e} / {err2:.2e} (per component {err_c:.2e})  loss {L:.8f} vs {L_ref:.8f}")
        assert err < GRAD_TOL and err2 < GRAD_TOL and err_c < COMPONENT_TOL
        assert abs(L - L_ref) < LOSS_TOL * abs(L_ref)
        assert np.abs(th - th1).max() < 1e-5 * max(1.0, np.abs(th1).max())


def test_pooled_sampler_with_distinct_picks_is_bit_reproducible_and_the_general_kernels_agree():
    d = dict(workload(3, 0.05).numpy(), pool_size=2048, pool_block=4096, pool_mode=1, pool_line=16, pool_segment=256)
    runs = []
    for tune in (None, None, {"pool_kernel": 0}):
        with make_nomad(d, SCATTER_DETERMINISTIC, tune=tune) as nm:
            assert nm.scatter_path() == (PATH_BINNED if tune else PATH_BINNED_POOLED)
            for t in range(4):
                nm.epoch(t)
            runs.append((nm.get_gradient(), nm.get_embedding()))
    assert np.array_equal(runs[0][0], runs[1][0]) and np.array_equal(runs[0][1], runs[1][1])
    assert np.abs(runs[0][0] - runs[2][0]).max() < 2e-5 * np.abs(runs[0][0]).max()       # another kernel, another summation order
    with pytest.raises(NomadError) as ei:                                                   # one sampling population only
        make_nomad(dict(small_random(6), pool_size=64, pool_block=256, pool_mode=1, pool_line=4, pool_segment=64), SCATTER_DETERMINISTIC)
    assert ei.value.code == -1


@pytest.mark.parametrize("mode", MODES)
def test_inverse_rank_weights_computed_by_the_library(mode):
    """edge_weights = NOMAD_WEIGHTS_INVERSE_RANK: p(j|i) from the position of j in i's row (Eq. 7 read with ranks from 1 and
    the row's own normaliser), on rows of different lengths; the oracle receives the same model as explicit weights."""
    from oracle import nomad_oracle as po
    d = dict(small_random(21, n=2500, groups=True, weights=False, s=3))
    deg = np.diff(d["row_ptr"])
    d["weights"] = np.concatenate([po.inverse_rank_weights(int(k)) for k in deg if k > 0]).astype(np.float32)
    assert deg.min() != deg.max()
    O = c_oracle.COracle(**d)
    _, g_ref, _ = O.epoch(d["theta0"], 0)
    L_ref = O.loss_and_grad(d["theta0"], 0, want_grad=False)[0]
    with make_nomad(dict(d, inverse_rank_weights=True), mode) as nm:
        assert abs(nm.loss(0) - L_ref) < LOSS_TOL * abs(L_ref)
        nm.epoch(0)
        assert grad_err(nm.get_gradient(), g_ref) < GRAD_TOL
    nm = Nomad(d["n"], d["n_clusters"], 3, 4.0, 5, 0.5, 1, mode, inverse_rank_weights=True)
    with pytest.raises(NomadError, match="INVALID_ARG"):                                    # weights and the rank model exclude each other
        nm.set_graph(d["row_ptr"], d["col_idx"], d["weights"], d["cluster_of"], d["cluster_group"])
    nm.close()


def test_pooled_sampler_is_bit_reproducible_and_needs_one_population():
    d = dict(workload(3, 0.05).numpy())
    d["pool_size"], d["pool_block"] = 2048, 4096
    runs = []
    for _ in range(2):
        with make_nomad(d, SCATTER_DETERMINISTIC) as nm:
            for t in range(4):
                nm.epoch(t)
            runs.append(nm.get_embedding())
    assert np.array_equal(runs[0], runs[1])
    g = small_random(6)
    g["pool_size"], g["pool_block"] = 64, 256
    with pytest.raises(NomadError) as ei:
        make_nomad(g, SCATTER_DETERMINISTIC)
    assert ei.value.code == -1


# ------------------------------------------------------------------ minibatch epochs
@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("case,B,pool", [("config1", 3, None), ("config3@0.05", 7, None), ("random-groups", 4, None),
                                         ("skewed", 5, None), ("config3@0.05", 6, (2048, 4096)), ("skewed", 50, (64, 1024))])
def test_minibatch_epoch_matches_the_oracle(case, B, pool, mode):
    """An epoch of B sequential sub-steps over head ranges: embedding after the epoch, gradient of the last
    sub-step, loss after it; then a second epoch from the GPU's embedding."""
    d = dict(skewed_degree_graph(8) if case == "skewed" else _case(case))
    d["batches_per_epoch"] = B
    if pool:
        d["pool_size"], d["pool_block"] = pool
    O = c_oracle.COracle(**d)
    th1, g_ref, _ = O.epoch(d["theta0"], 0)
    L_ref, _ = O.loss_and_grad(th1, 1, want_grad=False)
    with make_nomad(d, mode) as nm:
        nm.epoch(0)
        g, th, L = nm.get_gradient(), nm.get_embedding(), nm.loss(1)
        th2_ref, g2_ref, _ = O.epoch(th, 1)
        nm.epoch(1)
        g2, th2 = nm.get_gradient(), nm.get_embedding()
    scale = max(np.abs(g_ref).max(), 1e-30)
    note(f"  minibatch {case} B={B} pool={pool} mode={mode}: last-step grad err {np.abs(g - g_ref).max() / scale:.2e}, "
         f"theta err {np.abs(th - th1).max():.2e}")
    # the sub-steps compound fp32 differences of the earlier ones: compare against the size of a full-epoch gradient
    _, g_full = c_oracle.COracle(**{**d, "batches_per_epoch": 1}).loss_and_grad(d["theta0"], 0)
    assert np.abs(g - g_ref).max() < GRAD_TOL * max(np.abs(g_full).max(), scale)
    assert np.abs(th - th1).max() < 1e-5 * max(1.0, np.abs(th1).max())
    assert abs(L - L_ref) < LOSS_TOL * abs(L_ref)
    assert np.abs(th2 - th2_ref).max() < 1e-5 * max(1.0, np.abs(th2_ref).max())
    assert np.abs(g2 - g2_ref).max() < GRAD_TOL * max(np.abs(g_full).max(), np.abs(g2_ref).max())


def test_minibatch_epochs_are_bit_reproducible_and_one_batch_is_the_plain_epoch():
    d = dict(workload(3, 0.05).numpy())
    runs = []
    for B in (1, 1, 9, 9):
        d["batches_per_epoch"] = B
        with make_nomad(d, SCATTER_DETERMINISTIC) as nm:
            for t in range(3):
                nm.epoch(t)
            runs.append(nm.get_embedding())
    assert np.array_equal(runs[0], runs[1]) and np.array_equal(runs[2], runs[3])
    assert not np.array_equal(runs[0], runs[2])


# ------------------------------------------------------------------ degenerate and edge cases
@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("s", [0, 1, 4, 8, 9, 16])
def test_negative_counts_through_both_kernel_variants(s, mode):
    d = small_random(10 + s, n=1500, s=s, M=float(max(s, 2)))
    O = c_oracle.COracle(**d)
    _, g_ref, _ = O.epoch(d["theta0"], 0)
    with make_nomad(d, mode) as nm:
        if s:
            assert np.array_equal(nm.get_negatives(0), O.negatives(0))
        nm.epoch(0)
        assert grad_err(nm.get_gradient(), g_ref) < GRAD_TOL


@pytest.mark.parametrize("mode", MODES)
def test_empty_rows_empty_cluster_and_tiny_graphs(mode):
    # 6 points; points 4, 5 isolated; cluster 2 empty
    row_ptr = np.array([0, 2, 4, 6, 8, 8, 8], dtype=np.int32)
    col = np.array([1, 3, 0, 2, 1, 3, 0, 2], dtype=np.int32)
    d = dict(n=6, row_ptr=row_ptr, col_idx=col, weights=None, cluster_of=np.array([0, 0, 1, 1, 3, 3], dtype=np.int32),
             n_clusters=4, cluster_group=np.array([0, 0, 1, 1], dtype=np.int32), n_neg=5, noise_count=5.0, n_epochs=3,
             lr0=0.3, seed=5, theta0=np.array([[0, 0], [1, 0], [1, 1], [0, 1], [3, 3], [-2, 1]], dtype=np.float32))
    O = c_oracle.COracle(**d)
    th1, g_ref, _ = O.epoch(d["theta0"], 0)
    with make_nomad(d, mode) as nm:
        assert np.array_equal(nm.get_negatives(0), O.negatives(0))
        mu, counts = nm.get_means()
        assert counts.tolist() == [2, 2, 0, 2] and np.all(mu[2] == 0)
        nm.epoch(0)
        assert grad_err(nm.get_gradient(), g_ref) < GRAD_TOL
        assert abs(nm.loss(1) - O.loss_and_grad(th1, 1, want_grad=False)[0]) < 1e-5
    # a single point with no edge: the loss of an empty graph is 0 and nothing moves
    with Nomad(1, 1, 5, 5.0, 2, 1.0, 1, mode) as nm:
        nm.set_graph(np.zeros(2, np.int32), np.zeros(0, np.int32), None, np.zeros(1, np.int32))
        nm.set_embedding(np.array([[0.5, -1.0]], np.float32))
        nm.epoch(0)
        assert nm.loss(0) == 0.0 and np.array_equal(nm.get_embedding(), [[0.5, -1.0]])
        assert np.all(nm.get_gradient() == 0)


@pytest.mark.parametrize("mode", MODES)
def test_directed_graph_without_reverse_edges(mode):
    """The paper's kNN digraph is not symmetric; neither path may assume that it is."""
    d = small_random(50, n=2000, groups=False, weights=False, s=5, M=5.0)
    keep = np.random.default_rng(3).random(len(d["col_idx"])) < 0.6          # drop 40 % of the directed edges
    rows = np.repeat(np.arange(d["n"]), np.diff(d["row_ptr"]))
    d["col_idx"] = d["col_idx"][keep]
    d["row_ptr"] = np.concatenate([[0], np.cumsum(np.bincount(rows[keep], minlength=d["n"]))]).astype(np.int32)
    O = c_oracle.COracle(**d)
    _, g_ref, _ = O.epoch(d["theta0"], 0)
    with make_nomad(d, mode) as nm:
        nm.epoch(0)
        assert grad_err(nm.get_gradient(), g_ref) < GRAD_TOL


@pytest.mark.parametrize("mode", MODES)
def test_paper_graph_directed_with_inverse_rank_weights(mode):
    """Section 3.1's own input: the directed kNN graph (no transposed edges), p(j|i) from the inverse-rank model, Eq. 7."""
    d = workload(3, 0.03, paper_graph=True).numpy()
    assert d["weights"] is None and d["inverse_rank_weights"] and len(d["col_idx"]) == d["n"] * 15
    O = c_oracle.COracle(**d)
    _, g_ref, _ = O.epoch(d["theta0"], 0)
    with make_nomad(d, mode) as nm:
        assert np.array_equal(nm.get_negatives(0, 0, 4000), O.negatives(0)[:4000])
        assert abs(nm.loss(0) - O.loss_and_grad(d["theta0"], 0)[0]) < LOSS_TOL * abs(O.loss_and_grad(d["theta0"], 0)[0])
        nm.epoch(0)
        assert grad_err(nm.get_gradient(), g_ref) < GRAD_TOL
        th = nm.get_embedding()
        for t in range(1, 4):
            nm.epoch(t)
        th_ref = th.astype(np.float32)
        for t in range(1, 4):
            th_ref, g_ref, _ = O.epoch(th_ref, t)
        assert np.abs(nm.get_embedding() - th_ref).max() < 1e-5 * max(1.0, np.abs(th_ref).max())


def test_coincident_points_closed_form():
    """All rows equal: every q is 1, the loss is log(1+|M|) and no force acts (closed form, no oracle)."""
    d = small_random(30, groups=False, weights=False, s=5, M=5.0)
    d["theta0"] = np.full((d["n"], 2), 0.25, dtype=np.float32)
    with make_nomad(d, SCATTER_DETERMINISTIC) as nm:
        assert abs(nm.loss(0) - math.log(6.0)) < 1e-6
        nm.epoch(0)
        assert np.abs(nm.get_gradient()).max() < 1e-7


def test_forces_cancel_without_approximated_cells():
    d = workload(3, 0.05).numpy()
    with make_nomad(d, SCATTER_DETERMINISTIC) as nm:
        for t in range(3):
            nm.epoch(t)
        g = nm.get_gradient().astype(np.float64)
    assert np.abs(g.sum(0)).max() < 1e-4 * np.abs(g).sum(0).max()


def test_device_buffers_in_and_out():
    w = workload(3, 0.05)
    dev = torch.device("cuda:0")
    with Nomad(w.n, w.n_clusters, w.n_neg, w.noise_count, w.n_epochs, w.lr0, w.seed, SCATTER_DETERMINISTIC) as nm:
        nm.set_graph(w.row_ptr.to(dev), w.col_idx.to(dev), None, w.cluster_of.to(dev), None)
        nm.set_embedding(w.theta0.to(dev))
        nm.epoch(0)
        g_dev = nm.get_gradient(device=True)
        th_dev = nm.get_embedding(device=True)
        neg_dev = nm.get_negatives(0, 10, 500, device=True)
        assert g_dev.is_cuda and th_dev.is_cuda
        assert np.array_equal(g_dev.cpu().numpy(), nm.get_gradient())
        assert np.array_equal(th_dev.cpu().numpy(), nm.get_embedding())
        assert np.array_equal(neg_dev.cpu().numpy(), nm.get_negatives(0, 10, 500))


# ------------------------------------------------------------------ error paths (forced from the host)
def test_errors_are_codes_not_crashes():
    d = small_random(40, n=500)
    nm = Nomad(d["n"], d["n_clusters"], d["n_neg"], d["noise_count"], d["n_epochs"], d["lr0"], 1, SCATTER_DETERMINISTIC)
    with pytest.raises(NomadError, match="ORDER"):
        nm.epoch(0)
    with pytest.raises(NomadError, match="ORDER"):
        nm.set_embedding(d["theta0"])

    def bad(**over):
        a = dict(row_ptr=d["row_ptr"], col_idx=d["col_idx"], weights=d["weights"], cluster_of=d["cluster_of"],
                 cluster_group=d["cluster_group"])
        a.update(over)
        with pytest.raises(NomadError, match="BAD_GRAPH"):
            nm.set_graph(a["row_ptr"], a["col_idx"], a["weights"], a["cluster_of"], a["cluster_group"])

    rp = d["row_ptr"].copy(); rp[5], rp[6] = rp[6], rp[5] - 1
    bad(row_ptr=rp)
    rp = d["row_ptr"].copy(); rp[0] = 1
    bad(row_ptr=rp)
    col = d["col_idx"].copy(); col[3] = d["n"]
    bad(col_idx=col)
    col = d["col_idx"].copy(); col[0] = 0          # row 0 -> self loop
    bad(col_idx=col)
    w = d["weights"].copy(); w[10] = -1.0
    bad(weights=w)
    w = d["weights"].copy(); w[d["row_ptr"][3]:d["row_ptr"][4]] = 0.0
    bad(weights=w)
    cl = d["cluster_of"].copy(); cl[7] = d["n_clusters"]
    bad(cluster_of=cl)
    grp = d["cluster_group"].copy(); grp[1] = -2
    bad(cluster_group=grp)
    # after a failed set_graph the context has no graph
    with pytest.raises(NomadError, match="ORDER"):
        nm.epoch(0)
    nm.set_graph(d["row_ptr"], d["col_idx"], d["weights"], d["cluster_of"], d["cluster_group"])
    with pytest.raises(NomadError, match="ORDER"):
        nm.epoch(0)                                 # still no embedding
    nm.set_embedding(d["theta0"])
    with pytest.raises(NomadError, match="ORDER"):
        nm.get_gradient()
    with pytest.raises(NomadError, match="INVALID_ARG"):
        nm.epoch(d["n_epochs"])
    with pytest.raises(NomadError, match="INVALID_ARG"):
        nm.epoch(-1)
    with pytest.raises(NomadError, match="INVALID_ARG"):
        nm.get_negatives(0, 5, nm.num_edges() + 1)
    nm.epoch(0)
    nm.close()


# ------------------------------------------------------------------ sampled far field (opt-in variant of Eq. 5)
def _far_cases():
    yield "random-groups", dict(small_random(60, n=5000, s=3), sampled_far_field=True)
    yield "random-groups-s11", dict(small_random(61, n=3000, s=11, weights=False), sampled_far_field=True)      # run-time s path
    yield "config5@2e-3", dict(workload(5, 2e-3).numpy(), sampled_far_field=True)                                 # every cluster its own group
    yield "config4@5e-3-8groups", dict(workload(4, 5e-3, n_groups=8).numpy(), sampled_far_field=True)
    yield "no-groups", dict(small_random(62, groups=False, s=4), sampled_far_field=True)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("case", [c for c, _ in _far_cases()])
def test_sampled_far_field_matches_the_oracle(case, mode):
    d = dict(_far_cases())[case]
    note(f"sampled far field {case}")
    O = c_oracle.COracle(**d)
    with make_nomad(d, mode) as nm:
        E = len(d["col_idx"])
        assert np.array_equal(nm.get_negatives(2, 0, min(E, 20000)), O.negatives(2, 0, min(E, 20000)))
        L_ref, _ = O.loss_and_grad(d["theta0"], 1, want_grad=False)
        assert abs(nm.loss(1) - L_ref) < LOSS_TOL * abs(L_ref)
        th = np.asarray(d["theta0"], dtype=np.float32)
        for t in range(3):           # three epochs, each checked from the library's own embedding
            th_ref, g_ref, _ = O.epoch(th, t)
            nm.epoch(t)
            assert grad_err(nm.get_gradient(), g_ref) < GRAD_TOL, t
            th_new = nm.get_embedding()
            assert np.abs(th_new - th_ref).max() < 1e-5 * max(1.0, np.abs(th_ref).max())
            th = th_new
        A, B = nm.get_mean_field()
        assert not A.any() and not B.any()


def test_sampled_far_field_with_sub_steps_and_fallback_scatter():
    d = dict(small_random(63, n=4000, s=3), sampled_far_field=True, batches_per_epoch=4)
    O = c_oracle.COracle(**d)
    th_ref, g_ref, _ = O.epoch(d["theta0"], 0)
    for mode in (SCATTER_DETERMINISTIC, SCATTER_ATOMIC):
        with make_nomad(d, mode) as nm:
            nm.epoch(0)
            assert grad_err(nm.get_gradient(), g_ref) < GRAD_TOL
            assert np.abs(nm.get_embedding() - th_ref).max() < 1e-5


def test_sampled_far_field_estimates_the_exact_far_field_loss():
    """Averaged over the epochs' samples the sampled loss approaches the loss with Eq. 5 summed exactly (both have
    the same noise term in expectation; log is concave, so the sampled mean sits slightly below)."""
    d = workload(4, 5e-3, n_groups=8).numpy()
    rng = np.random.default_rng(5)
    d["theta0"] = (rng.normal(size=(d["n"], 2)) * 2.0).astype(np.float32)
    with make_nomad(d, SCATTER_DETERMINISTIC) as exact, make_nomad(dict(d, sampled_far_field=True), SCATTER_DETERMINISTIC) as far:
        L_exact = np.mean([exact.loss(t) for t in range(20)])
        L_far = np.mean([far.loss(t) for t in range(20)])
    note(f"loss with exact far field {L_exact:.5f}, sampled {L_far:.5f}")
    assert abs(L_far - L_exact) < 0.02 * L_exact


# ------------------------------------------------------------------ gradient through the cell means (opt-in)
def _mean_gradient_cases():
    yield "random-groups", dict(small_random(70, n=5000, s=3), mean_gradient=True)
    yield "random-groups-s11", dict(small_random(71, n=3000, s=11, weights=False), mean_gradient=True)          # run-time s path
    yield "config5@1e-3", dict(workload(5, 1e-3).numpy(), mean_gradient=True)                                    # every cluster its own group
    yield "config4@5e-3-8groups", dict(workload(4, 5e-3, n_groups=8).numpy(), mean_gradient=True)
    yield "no-groups", dict(small_random(72, groups=False, s=4), mean_gradient=True)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("case", [c for c, _ in _mean_gradient_cases()])
def test_gradient_through_the_means_matches_the_oracle(case, mode):
    d = dict(_mean_gradient_cases())[case]
    note(f"gradient through the means {case}")
    O = c_oracle.COracle(**d)
    g_const = None
    with make_nomad(d, mode) as nm:
        th = np.asarray(d["theta0"], dtype=np.float32)
        if case != "no-groups":                # spread the points so that the means' term is not negligible
            th = (np.random.default_rng(7).normal(size=th.shape) * 1.5).astype(np.float32)
            nm.set_embedding(th)
        for t in range(3):           # three epochs, each checked from the library's own embedding
            th_ref, g_ref, _ = O.epoch(th, t)
            nm.epoch(t)
            g = nm.get_gradient()
            assert grad_err(g, g_ref) < GRAD_TOL, t
            if d["cluster_group"] is not None:
                assert np.abs(g.astype(np.float64).sum(0)).max() < 1e-4 * np.abs(g_ref).max() * np.sqrt(d["n"])   # forces cancel
            th_new = nm.get_embedding()
            assert np.abs(th_new - th_ref).max() < 1e-5 * max(1.0, np.abs(th_ref).max())
            th = th_new
    if d["cluster_group"] is not None:         # and the term is there: the default gradient differs
        with make_nomad(dict(d, mean_gradient=False), mode) as nm:
            nm.set_embedding(th)
            nm.epoch(3)
            g_const = nm.get_gradient()
        _, g_ref, _ = O.epoch(th, 3)
        assert grad_err(g_const, g_ref) > 1e-4
