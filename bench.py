#!/usr/bin/env python3
"""Benchmark of the NOMAD epoch path on one MI355X.

A step is one nomad_epoch (cell means, [mean-field sums], edge pass, gradient scatter, SGD step)
over a synthetic kNN graph that is already resident in HBM.  Default workload: benchmark
configuration 4 (n = 10 M points, ~299 M directed edges, 5 negatives per edge).

Prints ONE JSON line:  metric = positive+negative edge updates per second, E * (1 + s) / t_epoch.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
FP32_VALU_PEAK_TFLOPS = 157.3  # MI355X published fp32 vector rate


MEAN_FIELD_FLOPS = 14.0        # per (head, cell): 2 differences, 1 + d^2 (4), reciprocal (1), p q (1), its sum (1),
                               # p q^2 (1), two multiply-adds for the derivative factor (4)


def algorithmic_bytes(kernel, n, E, s, R, grouped, weighted, deterministic, pool=None):
    """Bytes the method has to move per launch of each kernel, every gather / scatter counted at
    its useful size (8 B per embedding row, 4 B per index), an accumulation counted once.
    pool = (pool_size, pool_block) for the pooled sampler: the rows of the negatives are read and their
    forces handed on once per pool entry and block instead of once per negative."""
    w = 4 if weighted else 0
    mf = 12 if grouped else 0                    # A_i, B_i
    if kernel == "edges":
        per_edge = 4 + w + 8                     # col_idx, [p_e], theta_j
        per_edge += 4 if deterministic else 8    # a_e written / tail gradient accumulated
        if pool:
            negatives = (8 + 8) * pool[0] * ((E + pool[1] - 1) // pool[1])
        else:
            negatives = (8 + 8) * s * E          # theta_m read, the negatives' gradient contributions
        return per_edge * E + negatives + (4 + 8 + 8 + mf) * n   # row_ptr, theta_i, head gradient, [A,B]
    if kernel == "tiles":                        # accumulation of the binned forces (implementation traffic, not counted)
        return 24 * n                            # + the SGD step it takes: theta read and written, g written
    if kernel == "scatter":                      # fallback: combine of the fixed-point sums
        return (8 + 16 + 8) * n
    if kernel == "update":
        return 24 * n
    if kernel == "means":
        return 8 * n
    if kernel == "zero":
        return 8 * n
    if kernel == "mean_field":
        return (8 + 4 + 12) * n
    if kernel == "mean_gradient":                # per-edge coefficients read back, theta and the row sums of every head
        return 4 * E + (4 + 8 + 4 + 4) * n
    if kernel == "loss":
        return (4 + w + 8 + 8 * s) * E + (4 + 8 + mf) * n
    raise KeyError(kernel)


def measured_traffic(kernel, config, mode, launches_per_epoch=1.0, sampler="iid"):
    """(HBM bytes per launch, the kernel's milliseconds per epoch when the counters were read) from the committed rocprofv3
    counter summary (profiles/hbm_bytes_per_epoch.txt: lines `<config> <mode> <sampler> <kernel> <bytes of that kernel's
    launches of one epoch> <its ms per epoch in the kernel trace of the same build>`), or (None, None) if that kernel and
    workload have not been profiled.  The counters do not depend on how many launches an epoch's edge pass is cut into."""
    path = os.path.join(ROOT, "profiles", "hbm_bytes_per_epoch.txt")
    try:
        with open(path) as fh:
            for line in fh:
                f = line.split()
                if len(f) >= 5 and not line.startswith("#") and f[:4] == [f"config{config}", mode, sampler, kernel]:
                    return float(f[4]) / launches_per_epoch, (float(f[5]) if len(f) >= 6 else None)
    except OSError:
        pass
    return None, None


def attach_traffic(roofline, ms_per_epoch, config, mode, sampler="iid"):
    """roofline.traffic from the committed counters.  They are not read in this run: `traffic_current` says whether the
    kernel still takes the time it took when they were (within 15 %; small kernels: within 20 us), i.e. whether the
    summary under profiles/ still describes the kernel that was just timed."""
    traffic, ms_then = measured_traffic(roofline["kernel"], config, mode, roofline.get("launches_per_epoch", 1.0), sampler)
    roofline["traffic"] = traffic
    if traffic is not None and ms_then is not None:
        roofline["traffic_counted_at_ms_per_epoch"] = ms_then
        roofline["traffic_current"] = bool(abs(ms_per_epoch - ms_then) <= max(0.15 * ms_then, 0.02))


def copy_probe_gbs(torch, gib=4, steps=10):
    """Streaming copy of `gib` GiB with the library's probe kernel: read + write GB/s."""
    from paper_2505_15511_amd import binding
    src = torch.ones(gib << 28, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    binding.copy_probe(dst, src)
    torch.cuda.synchronize()
    ev0.record()
    for _ in range(steps):
        binding.copy_probe(dst, src)
    ev1.record()
    torch.cuda.synchronize()
    ms = ev0.elapsed_time(ev1) / steps
    nbytes = src.numel() * 4
    return dict(probe="copy", bytes_read=nbytes, bytes_written=nbytes, ms=ms, gbs_read_plus_write=2 * nbytes / ms / 1e6)


def _timed_probe(torch, launch, steps):
    """Average milliseconds of `launch()` over `steps` calls after one warm-up, by events on torch's current stream
    (the stream the probes are launched on)."""
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    issued = launch()
    torch.cuda.synchronize()
    ev0.record()
    for _ in range(steps):
        launch()
    ev1.record()
    torch.cuda.synchronize()
    return ev0.elapsed_time(ev1) / steps, issued


def gather_probe_glines(torch, table_mb=80, requests=1 << 30, steps=3):
    """Random 8-byte gathers over a table of `table_mb` MB (80 MB = the embedding at 10 M points): requests per
    second in units of 1e9.  Beyond the L2 size every request costs one 128-byte line, so this is also the line rate."""
    from paper_2505_15511_amd import binding
    table = torch.zeros(table_mb << 17, dtype=torch.float64, device="cuda")
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    ms, issued = _timed_probe(torch, lambda: binding.gather_probe(table, requests, sink), steps)
    return dict(probe="gather8", table_mb=table_mb, requests=issued, ms=ms, g_requests_per_s=issued / ms / 1e6)


def scatter_probe_rate(torch, kind, table_mb=80, requests=1 << 28, chains=1221, steps=3):
    from paper_2505_15511_amd import binding
    kinds = {"atomic_f32x2": binding.PROBE_ATOMIC_F32X2, "atomic_u64": binding.PROBE_ATOMIC_U64,
             "append12": binding.PROBE_APPEND12, "append12_grouped": binding.PROBE_APPEND12_GROUPED}
    if kind.startswith("append"):
        table = torch.zeros(int(requests * 12 * 1.3 + 256 * chains * 768) // 8 + 1, dtype=torch.float64, device="cuda")
    else:
        table = torch.zeros(table_mb << 17, dtype=torch.float64, device="cuda")
    ms, issued = _timed_probe(torch, lambda: binding.scatter_probe(kinds[kind], table, requests, chains), steps)
    out = dict(probe=kind, requests=issued, ms=ms, g_requests_per_s=issued / ms / 1e6)
    out.update(dict(chains_per_workgroup=chains) if kind.startswith("append") else dict(table_mb=table_mb))
    return out


def knn_index_run(args, torch, workloads):
    """nomad_knn_in_clusters on an equal-weight Gaussian mixture, clusters = components, data resident on the device.
    Reports point pairs per second of the whole call and the float32 matrix-core rate of its contraction."""
    from paper_2505_15511_amd import knn_in_clusters
    n, d, R, k = args.index_n, args.index_d, args.index_clusters, args.index_k
    X, c = workloads.gmm_points(n, d, R, 16.0, 4242, mix="equal", interleave=True)
    X, c = X.cuda(), c.cuda()
    torch.cuda.synchronize()
    times = []
    st = None
    for rep in range(args.warmup + args.steps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        out, st = knn_in_clusters(X, c, R, k, return_stats=True)
        torch.cuda.synchronize()
        if rep >= args.warmup:
            times.append(time.perf_counter() - t0)
    dt = sum(times) / len(times)
    flops = 2.0 * d * st["filter_pairs"]
    print(json.dumps({
        "metric": "in-cluster exact kNN, point pairs/sec at 1 GPU", "value": st["filter_pairs"] / dt, "unit": "pairs/s", "n_gpus": 1,
        "steps": len(times), "warmup": args.warmup, "ms_per_step": 1e3 * dt, "higher_is_better": True, "dtype": "f32 filter, f64 decision",
        "data": "synthetic",
        "config": {"workload": f"Gaussian mixture n={n}, d={d}, {R} equal clusters, k={k}"},
        "fallback_queries": st["fallback_queries"],
        "roofline": {"bound": "mfma", "kernel": "knn_filter (whole call timed: grouping, norms, filter, refinement)",
                     "achieved": flops / dt / 1e12, "peak": 157.3, "unit": "TFLOP/s", "frac": flops / dt / 1e12 / 157.3, "traffic": None}}))


def kmeans_index_run(args, torch, workloads):
    """nomad_kmeans_lloyd: --steps Lloyd iterations on a Gaussian mixture from centroids picked among the points."""
    from paper_2505_15511_amd import kmeans_lloyd
    n, d, K = args.index_n, args.index_d, args.index_clusters
    X, _ = workloads.gmm_points(n, d, K, 16.0, 4242, mix="equal", interleave=True)
    X = X.cuda()
    C0 = X[torch.randperm(n, generator=torch.Generator().manual_seed(1))[:K].cuda()].clone()
    kmeans_lloyd(X, C0, 1)                           # warm-up
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    C, labels, iters, inertia = kmeans_lloyd(X, C0, args.steps)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    flops = 2.0 * d * n * K * iters
    print(json.dumps({
        "metric": "K-Means Lloyd iterations, point-centroid pairs/sec at 1 GPU", "value": n * K * iters / dt, "unit": "pairs/s", "n_gpus": 1,
        "steps": iters, "warmup": 1, "ms_per_step": 1e3 * dt / iters, "higher_is_better": True, "dtype": "f32 filter, f64 decision",
        "data": "synthetic", "config": {"workload": f"Gaussian mixture n={n}, d={d}, K={K}"}, "inertia": inertia,
        "roofline": {"bound": "mfma", "kernel": "knn_filter (whole iteration timed: E step, sort, M step)",
                     "achieved": flops / dt / 1e12, "peak": 157.3, "unit": "TFLOP/s", "frac": flops / dt / 1e12 / 157.3, "traffic": None}}))


def metrics_run(args, torch, workloads):
    """The quality measures: random triplet accuracy over 10 triplets per point, neighbourhood preservation@15 on a
    seeded sample of 10,000 queries; the projection is a noisy linear one (the timing does not depend on it)."""
    from paper_2505_15511_amd import neighbourhood_preservation, random_triplet_accuracy
    n, d = args.index_n, args.index_d
    X, _ = workloads.gmm_points(n, d, args.index_clusters, 16.0, 4242, mix="equal", interleave=True)
    X = X.cuda()
    Y = (X[:, :2] + 0.5 * torch.randn(n, 2, generator=torch.Generator().manual_seed(2)).cuda()).contiguous()
    q = torch.randperm(n, generator=torch.Generator().manual_seed(3))[:10000].to(torch.int32).cuda()
    T = 10 * n
    random_triplet_accuracy(X, Y, 1000, 1)
    neighbourhood_preservation(X, Y, args.index_k, q[:256])
    torch.cuda.synchronize()
    times = {}
    for name, fn in (("triplets", lambda: random_triplet_accuracy(X, Y, T, 1)),
                     ("preservation", lambda: neighbourhood_preservation(X, Y, args.index_k, q))):
        best = None
        for _ in range(max(1, args.steps)):
            t0 = time.perf_counter()
            out = fn()
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            best = dt if best is None else min(best, dt)
        times[name] = (best, out)
    tb = 3.0 * (d + 2) * 4 * T                                    # three rows of each space per triplet
    print(json.dumps({
        "metric": "random triplets/sec at 1 GPU", "value": T / times["triplets"][0], "unit": "triplets/s", "n_gpus": 1,
        "steps": max(1, args.steps), "warmup": 1, "ms_per_step": 1e3 * times["triplets"][0], "higher_is_better": True, "dtype": "f64",
        "data": "synthetic", "config": {"workload": f"Gaussian mixture n={n}, d={d}; {T} triplets; preservation@{args.index_k} on 10000 queries"},
        "triplet_accuracy": times["triplets"][1][1], "preservation": times["preservation"][1][1],
        "preservation_ms": 1e3 * times["preservation"][0],
        "roofline": {"bound": "hbm", "kernel": "k_triplets (whole call timed)", "achieved": tb / times["triplets"][0] / 1e9, "peak": 8000.0,
                     "unit": "GB/s", "frac": tb / times["triplets"][0] / 8e12, "traffic": None}}))


def pca_run(args, torch, workloads):
    """nomad_pca_init on a Gaussian mixture; the contraction behind it is the covariance, n d^2 multiply-adds in float64."""
    from paper_2505_15511_amd import pca_init
    n, d = args.index_n, args.index_d
    X, _ = workloads.gmm_points(n, d, args.index_clusters, 16.0, 4242, mix="equal", interleave=True)
    X = X.cuda()
    pca_init(X, 1e-2)
    torch.cuda.synchronize()
    best, st = None, None
    for _ in range(max(1, args.steps)):
        t0 = time.perf_counter()
        _, st = pca_init(X, 1e-2, return_stats=True)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
    flops = 2.0 * n * d * d                                       # the full d x d covariance; the kernel computes one triangle of 64 x 64 tiles
    print(json.dumps({
        "metric": "PCA initialisation, points/sec at 1 GPU", "value": n / best, "unit": "points/s", "n_gpus": 1,
        "steps": max(1, args.steps), "warmup": 1, "ms_per_step": 1e3 * best, "higher_is_better": True, "dtype": "f64",
        "data": "synthetic", "config": {"workload": f"Gaussian mixture n={n}, d={d}"}, "solver": st,
        "roofline": {"bound": "mfma", "kernel": "k_pca_cov (whole call timed)", "achieved": flops / best / 1e12, "peak": 78.6,
                     "unit": "TFLOP/s", "frac": flops / best / 78.6e12, "traffic": None}}))


def pipeline_run(args, torch, workloads):
    """The composed method on --index-n points: partition, neighbours, graph, PCA start, --steps epochs, quality measures."""
    from paper_2505_15511_amd import pipeline
    n, d = args.index_n, args.index_d
    X, _ = workloads.gmm_points(n, d, args.index_clusters, 16.0, 4242, mix="dirichlet", interleave=True)
    X = X.cuda()
    pipeline.project(X[:20000].contiguous(), 16, n_epochs=2)          # warm-up: library load, torch's sort and unique
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    opts = {}
    if args.pool:                                                    # the opt-in pooled sampler for the epochs
        opts["pool_size"], opts["pool_block"] = (int(x) for x in args.pool.split(","))
    theta, info = pipeline.project(X, args.index_clusters, k=args.index_k, n_epochs=args.steps, seed=1, return_info=True, **opts)
    torch.cuda.synchronize()
    total = time.perf_counter() - t0
    t1 = time.perf_counter()
    preservation, accuracy = pipeline.evaluate(X, theta, k=args.index_k, seed=1)
    start_preservation, start_accuracy = pipeline.evaluate(X, info["theta0"], k=args.index_k, seed=1)
    t_eval = (time.perf_counter() - t1) / 2
    print(json.dumps({
        "metric": "points projected/sec at 1 GPU, whole method", "value": n / total, "unit": "points/s", "n_gpus": 1, "steps": args.steps,
        "warmup": 0, "ms_per_step": 1e3 * info["seconds"]["epochs"] / max(1, args.steps), "higher_is_better": True, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"Gaussian mixture n={n}, d={d}, {info['n_clusters']} clusters, k={args.index_k}, {args.steps} epochs, "
                               f"E={info['edges']} directed edges with inverse-rank weights"
                               + (f", pooled sampler {args.pool}" if args.pool else "")},
        "seconds": {**{k: round(v, 4) for k, v in info["seconds"].items()}, "total": round(total, 4), "evaluate": round(t_eval, 4)},
        "kmeans_iterations": info["kmeans_iterations"],
        "preservation_at_k": {"pca_start": start_preservation, "final": preservation},
        "triplet_accuracy": {"pca_start": start_accuracy, "final": accuracy}}))


def pool_of(w):
    """(pool size, block[, line, segment]) of a workload's pooled sampler, or None."""
    if not w.pool_size:
        return None
    return (w.pool_size, w.pool_block, w.pool_line, w.pool_segment, w.pool_mode) if w.pool_mode else (w.pool_size, w.pool_block)


def timed_epochs(torch, w, mode, steps, warmup, batches=1, phases=0, tune=None):
    """`warmup` untimed and `steps` timed epochs of workload w (graph and embedding resident on the device before the
    clock starts), with the library's per-launch HIP events on its stream.  Returns the timings, the per-kernel
    figures per epoch and the roofline entry of the kernel that takes most of the epoch."""
    from paper_2505_15511_amd import Nomad, SCATTER_DETERMINISTIC, binding
    dev = "cuda"
    n, E, s, R = w.n, w.n_edges, w.n_neg, w.n_clusters
    pool = pool_of(w)
    nm = Nomad(n, R, s, w.noise_count, w.n_epochs, w.lr0, w.seed, mode, pool_size=w.pool_size, pool_block=w.pool_block,
               batches_per_epoch=batches, sampled_far_field=w.sampled_far_field, mean_gradient=w.mean_gradient,
               pool_mode=w.pool_mode, pool_line=w.pool_line, pool_segment=w.pool_segment,
               inverse_rank_weights=w.inverse_rank_weights, tune=dict(({"record_phases": phases} if phases else {}), **(tune or {})) or None)
    t0 = time.time()
    nm.set_graph(w.row_ptr.to(dev), w.col_idx.to(dev), None if w.weights is None else w.weights.to(dev), w.cluster_of.to(dev),
                 None if w.cluster_group is None else w.cluster_group.to(dev))
    nm.set_embedding(w.theta0.to(dev))
    torch.cuda.synchronize()
    setup_s = time.time() - t0
    for t in range(warmup):
        nm.epoch(t)
    torch.cuda.synchronize()
    nm.profile(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(warmup, warmup + steps):
        nm.epoch(t)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = nm.profile_read()
    nm.profile(False)
    loss = nm.loss(warmup + steps)
    path_name, state_gb, note = binding.PATH_NAMES[nm.scatter_path()], nm.device_bytes() / 1e9, nm.note()
    nm.close()
    grouped = w.cluster_group is not None
    weighted = w.weights is not None or w.inverse_rank_weights
    det = mode == SCATTER_DETERMINISTIC
    kernels = {}
    for name, (ms, cnt) in prof.items():
        if cnt:
            ab = algorithmic_bytes(name, n, E, s, R, grouped, weighted, det, pool)
            # per epoch: with record phases an epoch's edge pass is several launches, each over its share of the edges
            kernels[name] = dict(ms=ms / steps, launches=cnt, launches_per_epoch=cnt / steps, algorithmic_gb=ab / 1e9,
                                 gbs=ab / (ms / steps) / 1e6)
    dom = max(kernels, key=lambda k: kernels[k]["ms"])
    if dom in ("mean_field", "mean_gradient"):
        # n * |R| kernel evaluations (Eq. 5 and its derivative factor): plain-ALU bound, not HBM bound
        flops = MEAN_FIELD_FLOPS * float(n) * float(R)
        roofline = dict(bound="alu", kernel=dom, achieved=flops / (kernels[dom]["ms"] * 1e-3) / 1e12,
                        peak=FP32_VALU_PEAK_TFLOPS, unit="TFLOP/s", traffic=None)
    else:
        # per launch: an epoch's edge pass is `launches_per_epoch` launches (record phases), each over its share of the edges
        lpe = kernels[dom]["launches_per_epoch"]
        roofline = dict(bound="hbm", kernel=dom, achieved=kernels[dom]["gbs"], peak=HBM_PEAK_GBS, unit="GB/s", traffic=None,
                        launches_per_epoch=lpe, algorithmic_gb_per_launch=round(kernels[dom]["algorithmic_gb"] / lpe, 3),
                        ms_per_launch=round(kernels[dom]["ms"] / lpe, 4))
    roofline["frac"] = roofline["achieved"] / roofline["peak"]
    epoch_bytes = sum(algorithmic_bytes(k, n, E, s, R, grouped, weighted, det, pool) for k in kernels
                      if k not in ("mean_field", "mean_gradient"))
    return dict(ms_per_step=1e3 * elapsed / steps, elapsed=elapsed, kernels=kernels, roofline=roofline, loss=loss, path=path_name,
                state_gb=state_gb, note=note, setup_s=setup_s, grouped=grouped, epoch_bytes=epoch_bytes)


def summary_of(w, m, steps):
    """The short form of a measurement for the lists of variants and configurations."""
    E, s = w.n_edges, w.n_neg
    t = m["elapsed"] / steps
    return {"workload": w.name, "n": w.n, "edges": E, "ms_per_step": round(1e3 * t, 4), "edges_per_s": E / t, "updates_per_s": E * (1 + s) / t,
            "kernels_ms": {k: round(v["ms"], 4) for k, v in m["kernels"].items()}, "scatter_path": m["path"],
            "library_state_gb": round(m["state_gb"], 2),
            "roofline": {k: (round(v, 4) if isinstance(v, float) else v) for k, v in m["roofline"].items()}, "frac": round(m["roofline"]["frac"], 4)}


def hip_graph_run(args, torch, Nomad, w, mode, warmup, steps):
    """The timed epochs recorded once into a HIP graph (nomad_epoch only enqueues kernels on the caller's stream) and
    replayed: one graph launch for 2 x steps kernels."""
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        nm = Nomad.from_workload(w, mode, stream=side.cuda_stream, batches_per_epoch=args.batches)
        for t in range(warmup):
            nm.epoch(t)
        side.synchronize()
        theta_w = nm.get_embedding(device=True).clone()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for t in range(warmup, warmup + steps):
                nm.epoch(t)
        best = float("inf")
        for _ in range(5):
            nm.set_embedding(theta_w)
            side.synchronize()
            t0 = time.perf_counter()
            graph.replay()
            side.synchronize()
            best = min(best, time.perf_counter() - t0)
        nm.set_embedding(theta_w)
        side.synchronize()
        t0 = time.perf_counter()
        for t in range(warmup, warmup + steps):
            nm.epoch(t)
        side.synchronize()
        eager = time.perf_counter() - t0
        E, s = w.n_edges, w.n_neg
        print(json.dumps({"metric": "positive+negative edge updates/sec per epoch at 1 GPU", "value": E * (1 + s) / (best / steps),
                          "unit": "updates/s", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": 1e3 * best / steps,
                          "ms_per_step_eager_launches": 1e3 * eager / steps, "higher_is_better": True, "dtype": "f32",
                          "data": "synthetic", "config": {"workload": w.name, "launch": f"{steps} epochs replayed as one HIP graph"}}))
        nm.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, help="benchmark configuration 1-5")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the configuration (testing only)")
    ap.add_argument("--mode", choices=["det", "atomic"], default="det")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="the default run only: skip the variants and the other configurations")
    ap.add_argument("--groups", type=int, default=None, help="deal the clusters into this many groups")
    ap.add_argument("--pool", default=None, metavar="P,G",
                    help="opt-in pooled sampler: pool size and block length (e.g. 2048,4096), or P,G,line,segment for the "
                         "sampler with distinct picks (e.g. 4096,8192,16,256; a fifth value 2 selects stratified pools); not the benchmark's sampler")
    ap.add_argument("--graph", choices=["symmetrised", "paper"], default="symmetrised",
                    help="paper: the directed kNN graph with inverse-rank weights of Section 3.1 / Eq. 7 (planted configs); "
                         "the benchmark uses the symmetrised unit-weight graph")
    ap.add_argument("--far-field", choices=["exact", "sampled"], default="exact",
                    help="sampled: estimate Eq. 5's sum over the approximated cells from the samples (opt-in variant; "
                         "grouped configurations); the benchmark sums it exactly")
    ap.add_argument("--hip-graph", action="store_true",
                    help="record the timed epochs into one HIP graph on a side stream and time its replay (shows what the "
                         "launch-bound small configurations cost without per-kernel launches; prints a reduced line)")
    ap.add_argument("--mean-gradient", action="store_true",
                    help="let the gradient flow through the cell means (opt-in; grouped configurations); the benchmark "
                         "holds them constant within an epoch")
    ap.add_argument("--index", choices=["knn", "kmeans", "metrics", "pca", "pipeline"], default=None,
                    help="knn: time nomad_knn_in_clusters (the upstream index of Section 3.2) on a Gaussian mixture of "
                         "--index-n points in --index-d dimensions and --index-clusters clusters instead of the epoch path")
    ap.add_argument("--index-n", type=int, default=1_000_000)
    ap.add_argument("--index-d", type=int, default=128)
    ap.add_argument("--index-clusters", type=int, default=256)
    ap.add_argument("--index-k", type=int, default=15)
    ap.add_argument("--phases", type=int, default=0, help="record phases of the deterministic edge pass (0: the library's choice)")
    ap.add_argument("--tune", action="append", default=[], metavar="KNOB=VALUE",
                    help="a launch-shape knob of nomad_tune by its name in binding.TUNE (edge_block, workgroups_per_cu, record_sort, "
                         "flush_rounds, ...); may be given several times")
    ap.add_argument("--batches", type=int, default=1, help="sub-steps per epoch (minibatch epochs); the benchmark uses 1")
    ap.add_argument("--probe", choices=["copy", "gather", "atomic_f32x2", "atomic_u64", "append12", "append12_grouped", "limits"], default=None,
                    help="run only one memory-system probe: streaming copy (counter calibration / practical HBM ceiling), "
                         "random 8-byte gathers or atomics over a table of --probe-mb MB, or 12-byte record appends to "
                         "--probe-chains chains per workgroup; limits: the whole table (gathers over 1 MB .. 2 GB, atomics, appends)")
    ap.add_argument("--probe-mb", type=int, default=80)
    ap.add_argument("--probe-chains", type=int, default=1221)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build covers one GPU's share of the path; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2505_15511_amd import Nomad, SCATTER_ATOMIC, SCATTER_DETERMINISTIC, binding, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda"
    if args.probe == "copy":
        print(json.dumps(copy_probe_gbs(torch, steps=args.steps)))
        return
    if args.probe == "limits":
        rows = [copy_probe_gbs(torch, steps=5)]
        rows += [gather_probe_glines(torch, table_mb=mb, steps=3) for mb in (1, 4, 16, 64, 80, 160, 512, 2048)]
        rows += [scatter_probe_rate(torch, k, table_mb=80, steps=2) for k in ("atomic_f32x2", "atomic_u64")]
        rows += [scatter_probe_rate(torch, "append12", chains=c, steps=3) for c in (64, 611, 1221, 7324)]
        rows += [scatter_probe_rate(torch, "append12_grouped", chains=c, steps=3) for c in (1221, 7324)]
        print(json.dumps({"memory_system_limits": rows}))
        return
    if args.probe == "gather":
        print(json.dumps(gather_probe_glines(torch, table_mb=args.probe_mb, steps=min(args.steps, 5))))
        return
    if args.probe:
        print(json.dumps(scatter_probe_rate(torch, args.probe, table_mb=args.probe_mb, chains=args.probe_chains, steps=min(args.steps, 5))))
        return
    if args.index == "knn":
        return knn_index_run(args, torch, workloads)
    if args.index == "kmeans":
        return kmeans_index_run(args, torch, workloads)
    if args.index == "metrics":
        return metrics_run(args, torch, workloads)
    if args.index == "pca":
        return pca_run(args, torch, workloads)
    if args.index == "pipeline":
        return pipeline_run(args, torch, workloads)
    t0 = time.time()
    w = workloads.make_config(args.config, scale=args.scale, device=dev if args.config >= 3 else "cpu",
                              n_groups=args.groups, paper_graph=args.graph == "paper")
    torch.cuda.synchronize()
    gen_s = time.time() - t0
    pool = None
    if args.pool:
        pool = tuple(int(x) for x in args.pool.split(","))
        w.pool_size, w.pool_block = pool[:2]
        if len(pool) >= 4:                      # points per pool line, segment[, mode]: the sampler with distinct picks
            w.pool_mode, w.pool_line, w.pool_segment = (pool[4] if len(pool) == 5 else 1), pool[2], pool[3]
    n, E, s, R = w.n, w.n_edges, w.n_neg, w.n_clusters
    steps, warmup = args.steps, args.warmup
    if warmup + steps > w.n_epochs:
        steps = max(1, w.n_epochs - warmup)
    mode = SCATTER_DETERMINISTIC if args.mode == "det" else SCATTER_ATOMIC
    w.sampled_far_field = args.far_field == "sampled"
    w.mean_gradient = args.mean_gradient
    if args.hip_graph:
        return hip_graph_run(args, torch, Nomad, w, mode, warmup, steps)
    default_run = (args.config == 4 and args.scale == 1.0 and args.mode == "det" and pool is None and args.groups is None and
                   args.batches == 1 and args.graph == "symmetrised" and not w.sampled_far_field and not w.mean_gradient and
                   args.phases == 0 and not args.tune)
    m = timed_epochs(torch, w, mode, steps, warmup, batches=args.batches, phases=args.phases,
                     tune={kv.split('=')[0]: int(kv.split('=')[1]) for kv in args.tune})
    kernels, roofline, loss, elapsed, epoch_bytes = m["kernels"], m["roofline"], m["loss"], m["elapsed"], m["epoch_bytes"]
    ms_per_step, path_name, state_gb, setup_s, grouped = m["ms_per_step"], m["path"], m["state_gb"], m["setup_s"], m["grouped"]
    dom = roofline["kernel"]
    if args.scale == 1.0 and args.groups is None and pool is None and args.batches == 1 and args.graph == "symmetrised" \
            and not w.sampled_far_field and not w.mean_gradient:
        attach_traffic(roofline, kernels[dom]["ms"], args.config, args.mode)
    out = {
        "metric": "positive+negative edge updates/sec per epoch at 1 GPU",
        "value": E * (1 + s) / (elapsed / steps),
        "unit": "updates/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: n={n}, E={E} directed edges, |R|={R} clusters, s={s} negatives/edge, "
                               f"|M|={w.noise_count:g}, {'grouped (mean-field)' if grouped else 'no approximated cells'}",
                   "scatter_mode": args.mode,
                   "batches_per_epoch": args.batches,
                   "sampler": "iid per edge" if pool is None else f"pooled, {pool[0]} points per block of {pool[1]} edges (opt-in variant)"
                              + (f", distinct picks, lines of {pool[2]} points, segments of {pool[3]} positions" if len(pool) >= 4 else "")
                              + (", stratified pools" if len(pool) == 5 and pool[4] == 2 else ""),
                   "scatter_path": None,
                   "far_field": "Eq. 5 summed over the approximated cells" if not w.sampled_far_field else
                                "estimated from the samples (opt-in variant)",
                   "means": "constants of the epoch" if not w.mean_gradient else "differentiated (opt-in variant)"},
        "edges_per_sec": E / (elapsed / steps),
        "epoch_model_gb": epoch_bytes / 1e9,
        "epoch_hbm_frac_model": epoch_bytes / (elapsed / steps) / 1e9 / HBM_PEAK_GBS,
        "kernels_ms": {k: round(v["ms"], 4) for k, v in kernels.items()},
        "launches_per_epoch": {k: v["launches_per_epoch"] for k, v in kernels.items()},
        "loss_after": loss,
        "setup_s": round(setup_s, 3), "generate_s": round(gen_s, 3),
        "library_state_gb": round(state_gb, 2),
        "roofline": roofline,
    }
    out["config"]["scatter_path"] = path_name
    out["copy_probe_gbs"] = round(copy_probe_gbs(torch, gib=2, steps=5)["gbs_read_plus_write"], 1)
    # the rate at which this machine serves independent 8-byte gathers from a table the size of the embedding at
    # 10 M points: E * s such gathers per epoch bound the i.i.d. sampler's edge pass from below (E s / rate)
    gp = gather_probe_glines(torch, table_mb=80, steps=3)
    out["gather_probe_glines"] = round(gp["g_requests_per_s"], 2)
    out["gather_probe"] = {"table_mb": 80, "requests": gp["requests"], "ms": round(gp["ms"], 3),
                           "floor_ms_for_this_workload": round(E * s / gp["g_requests_per_s"] / 1e6, 2) if pool is None and s else None}

    if not args.no_cpu_baseline:
        from oracle import c_oracle
        d = w.numpy()
        O = c_oracle.COracle(**d)
        if grouped and not w.sampled_far_field and float(n) * R > 2e10:
            # the full mean-field sum is out of reach on the host: loss + gradient terms of 1/64 of the heads
            # (a contiguous range in the middle: every head pays the same |R| cell evaluations), extrapolated
            h0 = n // 2
            h1 = h0 + max(1, n // 64)
            t0 = time.perf_counter()
            O.loss_and_grad(d["theta0"], 0, head_range=(h0, h1))
            dt = time.perf_counter() - t0
            frac = (h1 - h0) / float(n)
            cpu = dict(value=E * (1 + s) * frac / dt, unit="updates/s", cores=O.threads, kind="oracle",
                       sample=f"loss+gradient terms of the heads {h0}..{h1 - 1} of {w.name} (1/{round(1 / frac)} of the heads, "
                              f"each with its full sum over the cells) in {dt:.1f} s; value extrapolated to the whole epoch")
        else:
            reps, dt = 0, 0.0
            t0 = time.perf_counter()
            while dt < 5.0 and reps < 1000:      # small workloads: repeat the epoch until the sample is measurable
                O.loss_and_grad(d["theta0"], reps)
                reps += 1
                dt = time.perf_counter() - t0
            cpu = dict(value=reps * E * (1 + s) / dt, unit="updates/s", cores=O.threads, kind="oracle",
                       sample=f"{reps} full epoch(s) of loss+gradient of {w.name} ({E} edges each) in {dt:.2f} s")
        out["cpu_baseline"] = cpu
    if default_run and not args.no_extras:
        # Beside the headline (which stays the i.i.d. sampler): the pooled sampler with distinct picks on the same workload,
        # priced with its own algorithmic bytes, and the other configurations (deterministic) plus configuration 4 on the
        # atomic path, five timed epochs each.
        out["variants"] = {}
        for key, pmode, text in (("pooled_exact", 1, "the negatives of one edge are i.i.d. uniform, negatives of different edges of a block are "
                                                       "not independent"),
                                 ("pooled_stratified", 2, "as pooled_exact with the pools' lines dealt from a permutation of the lines of points: "
                                                          "every point is a pool member equally often; the negatives of one edge are drawn "
                                                          "without replacement at line granularity")):
            psize = 2048 if pmode == 1 else 4096
            w.pool_size, w.pool_block, w.pool_mode, w.pool_line, w.pool_segment = psize, 8192, pmode, 16, 256
            mv = timed_epochs(torch, w, SCATTER_DETERMINISTIC, 10, 3)
            attach_traffic(mv["roofline"], mv["kernels"][mv["roofline"]["kernel"]]["ms"], 4, "det", key)
            out["variants"][key] = dict(summary_of(w, mv, 10), sampler=f"pooled, distinct picks: {psize} points in lines of 16 per block of 8192 "
                                        "positions dealt in segments of 256; " + text + " (opt-in variant)")
        w.pool_size, w.pool_block, w.pool_mode, w.pool_line, w.pool_segment = 0, 0, 0, 1, 64
        ma = timed_epochs(torch, w, SCATTER_ATOMIC, 5, 2)
        attach_traffic(ma["roofline"], ma["kernels"][ma["roofline"]["kernel"]]["ms"], 4, "atomic")
        out["all_configs"] = {"4_atomic": summary_of(w, ma, 5)}
        del w
        torch.cuda.empty_cache()
        for cfg in (1, 2, 3, 5):
            wc = workloads.make_config(cfg, device=dev if cfg >= 3 else "cpu")
            torch.cuda.synchronize()
            mc = timed_epochs(torch, wc, SCATTER_DETERMINISTIC, 5, 2)
            if mc["roofline"]["bound"] == "hbm":
                attach_traffic(mc["roofline"], mc["kernels"][mc["roofline"]["kernel"]]["ms"], cfg, "det")
            out["all_configs"][str(cfg)] = summary_of(wc, mc, 5)
            del wc, mc
            torch.cuda.empty_cache()
        out["all_configs"]["4"] = {"ms_per_step": round(ms_per_step, 4), "edges_per_s": out["edges_per_sec"], "updates_per_s": out["value"],
                                   "frac": round(roofline["frac"], 4)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
