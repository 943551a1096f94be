"""Thin ctypes binding of libnomad's C ABI (include/nomad.h).

Argument marshalling only: every step of the epoch runs in the library's HIP kernels.  Buffers
may be torch tensors (CPU or on the context's GPU) or numpy arrays; torch is used here for
device memory and stream handles, nothing else.  There is no CPU fallback: if the shared library
has not been built, loading fails with an error."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import _build

NOMAD_HOST, NOMAD_DEVICE = 0, 1
SCATTER_DETERMINISTIC, SCATTER_ATOMIC = 0, 1
FAR_FIELD_EXACT, FAR_FIELD_SAMPLED = 0, 1
K_MEANS, K_MEANFIELD, K_EDGES, K_SCATTER, K_UPDATE, K_LOSS, K_ZERO, K_TILES = range(8)
KERNEL_NAMES = ["means", "mean_field", "edges", "scatter", "update", "loss", "zero", "tiles", "mean_gradient"]
ERRORS = {-1: "NOMAD_E_INVALID_ARG", -2: "NOMAD_E_BAD_GRAPH", -3: "NOMAD_E_ORDER", -4: "NOMAD_E_TOO_LARGE",
          -5: "NOMAD_E_OOM", -6: "NOMAD_E_HIP"}

EXPORTS = ["nomad_create", "nomad_destroy", "nomad_set_graph", "nomad_set_embedding", "nomad_epoch", "nomad_loss",
           "nomad_get_embedding", "nomad_get_gradient", "nomad_get_negatives", "nomad_get_means",
           "nomad_get_mean_field", "nomad_num_edges", "nomad_scatter_path", "nomad_device_bytes", "nomad_tune", "nomad_profile", "nomad_profile_read", "nomad_last_error",
           "nomad_copy_probe", "nomad_gather_probe", "nomad_scatter_probe", "nomad_knn_in_clusters", "nomad_kmeans_lloyd", "nomad_neighbourhood_preservation",
           "nomad_random_triplet_accuracy", "nomad_random_triplet_accuracy_noalloc", "nomad_pca_init", "nomad_kmeans_lsh_init"]


class NomadConfig(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("n_points", C.c_int64), ("n_clusters", C.c_int32), ("n_neg", C.c_int32),
                ("noise_count", C.c_float), ("n_epochs", C.c_int32), ("lr0", C.c_float), ("seed", C.c_uint64),
                ("scatter_mode", C.c_int32), ("batches_per_epoch", C.c_int32), ("device", C.c_int32),
                ("stream", C.c_void_p), ("pool_size", C.c_int32), ("pool_block", C.c_int32), ("far_field", C.c_int32),
                ("mean_gradient", C.c_int32), ("pool_mode", C.c_int32), ("pool_line", C.c_int32), ("pool_segment", C.c_int32),
                ("edge_weights", C.c_int32)]


PATH_ATOMIC_FP32, PATH_BINNED, PATH_BINNED_POOLED, PATH_FIXED_ATOMICS = 1, 2, 3, 4
PATH_NAMES = {0: "none", 1: "atomic_fp32", 2: "binned", 3: "binned_pooled", 4: "fixed_point_atomics"}
TUNE = {"edge_block": 1, "workgroups_per_cu": 2, "scatter_path": 3, "pool_kernel": 4, "record_phases": 5, "record_sort": 6, "flush_rounds": 7}
POOL_PICKS16, POOL_DISTINCT, POOL_STRATIFIED = 0, 1, 2


class NomadError(RuntimeError):
    def __init__(self, code, text=""):
        self.code = code
        super().__init__(f"{ERRORS.get(code, code)}: {text}")


_lib = None


def load_library():
    """dlopen libnomad.so.  Raises if it has not been built (run __graft_entry__.build())."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB_PATH):
        raise RuntimeError(f"{_build.LIB_PATH} is missing: build the HIP library first "
                           "(python -c 'import __graft_entry__ as g; g.build()'); there is no fallback path")
    # torch (the harness's source of device memory and streams) brings its own copy of the HIP runtime: load it
    # first, so that this process ends up with one runtime and libnomad.so binds to the one torch allocates with
    import torch  # noqa: F401
    lib = C.CDLL(_build.LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.nomad_create.argtypes = [C.POINTER(NomadConfig), C.POINTER(vp)]
    lib.nomad_destroy.argtypes = [vp]
    lib.nomad_destroy.restype = None
    lib.nomad_set_graph.argtypes = [vp, vp, vp, vp, vp, vp, C.c_int]
    lib.nomad_set_embedding.argtypes = [vp, vp, C.c_int]
    lib.nomad_epoch.argtypes = [vp, i32]
    lib.nomad_loss.argtypes = [vp, i32, C.POINTER(C.c_double)]
    lib.nomad_get_embedding.argtypes = [vp, vp, C.c_int]
    lib.nomad_get_gradient.argtypes = [vp, vp, C.c_int]
    lib.nomad_get_negatives.argtypes = [vp, i32, i64, i64, vp, C.c_int]
    lib.nomad_get_means.argtypes = [vp, vp, vp, C.c_int]
    lib.nomad_get_mean_field.argtypes = [vp, vp, vp, C.c_int]
    lib.nomad_num_edges.argtypes = [vp]
    lib.nomad_num_edges.restype = i64
    lib.nomad_scatter_path.argtypes = [vp]
    lib.nomad_device_bytes.argtypes = [vp]
    lib.nomad_device_bytes.restype = i64
    lib.nomad_tune.argtypes = [vp, C.c_int, C.c_int]
    lib.nomad_profile.argtypes = [vp, C.c_int]
    lib.nomad_profile_read.argtypes = [vp, C.c_int, C.POINTER(C.c_double), C.POINTER(i64)]
    lib.nomad_copy_probe.argtypes = [vp, vp, C.c_uint64, vp]
    lib.nomad_gather_probe.argtypes = [vp, C.c_uint64, C.c_uint64, C.POINTER(C.c_uint64), vp, vp]
    lib.nomad_scatter_probe.argtypes = [C.c_int, vp, C.c_uint64, C.c_uint64, C.c_uint32, C.POINTER(C.c_uint64), vp]
    lib.nomad_knn_in_clusters.argtypes = [vp, i64, i32, vp, i32, i32, vp, C.c_int, i32, vp, vp]
    lib.nomad_kmeans_lloyd.argtypes = [vp, i64, i32, i32, vp, i32, vp, C.POINTER(i32), C.POINTER(C.c_double), C.c_int, i32, vp]
    lib.nomad_neighbourhood_preservation.argtypes = [vp, i64, i32, vp, i32, i32, vp, i64, C.POINTER(i64), C.c_int, i32, vp]
    lib.nomad_random_triplet_accuracy.argtypes = [vp, i64, i32, vp, i32, i64, C.c_uint64, C.POINTER(i64), C.c_int, i32, vp]
    lib.nomad_random_triplet_accuracy_noalloc.argtypes = [vp, i64, i32, vp, i32, i64, C.c_uint64, C.POINTER(i64), i32, vp]
    lib.nomad_pca_init.argtypes = [vp, i64, i32, C.c_float, vp, C.POINTER(C.c_double), C.c_int, i32, vp]
    lib.nomad_kmeans_lsh_init.argtypes = [vp, i64, i32, i32, vp, vp, i32, vp, vp, C.c_int, i32, vp]
    lib.nomad_last_error.argtypes = [vp]
    lib.nomad_last_error.restype = C.c_char_p
    _lib = lib
    return lib


def _is_torch(x):
    return x is not None and type(x).__module__.startswith("torch")


def _marshal(x, np_dtype, count=None):
    """-> (pointer, mem, keepalive).  Accepts None, torch tensor (cpu/cuda) or array-like."""
    if x is None:
        return None, None, None
    if _is_torch(x):
        import torch
        want = {np.int32: torch.int32, np.float32: torch.float32, np.int64: torch.int64}[np_dtype]
        t = x if (x.dtype == want and x.is_contiguous()) else x.to(want).contiguous()
        if count is not None and t.numel() != count:
            raise ValueError(f"expected {count} elements, got {t.numel()}")
        return C.c_void_p(t.data_ptr()), (NOMAD_DEVICE if t.is_cuda else NOMAD_HOST), t
    a = np.ascontiguousarray(x, dtype=np_dtype)
    if count is not None and a.size != count:
        raise ValueError(f"expected {count} elements, got {a.size}")
    return a.ctypes.data_as(C.c_void_p), NOMAD_HOST, a


def copy_probe(dst, src, stream=None):
    """Enqueue the library's streaming copy kernel between two device tensors of equal size."""
    import torch
    lib = load_library()
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes and src.is_cuda and dst.is_cuda
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    rc = lib.nomad_copy_probe(C.c_void_p(dst.data_ptr()), C.c_void_p(src.data_ptr()), nbytes, C.c_void_p(stream or None))
    if rc:
        raise NomadError(rc, "nomad_copy_probe")


PROBE_ATOMIC_F32X2, PROBE_ATOMIC_U64, PROBE_APPEND12, PROBE_APPEND12_GROUPED = 1, 2, 3, 4


def gather_probe(table, n_requests, sink, stream=None):
    """Enqueue nomad_gather_probe on a device tensor `table`; returns the number of requests issued."""
    import torch
    lib = load_library()
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    issued = C.c_uint64(0)
    rc = lib.nomad_gather_probe(C.c_void_p(table.data_ptr()), table.numel() * table.element_size(), int(n_requests), C.byref(issued),
                                C.c_void_p(sink.data_ptr()), C.c_void_p(stream or None))
    if rc:
        raise NomadError(rc, "nomad_gather_probe")
    return int(issued.value)


def scatter_probe(kind, table, n_requests, chains=1, stream=None):
    """Enqueue nomad_scatter_probe (atomics or appends) on a device tensor `table`; returns the requests issued."""
    import torch
    lib = load_library()
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    issued = C.c_uint64(0)
    rc = lib.nomad_scatter_probe(int(kind), C.c_void_p(table.data_ptr()), table.numel() * table.element_size(), int(n_requests),
                                 int(chains), C.byref(issued), C.c_void_p(stream or None))
    if rc:
        raise NomadError(rc, "nomad_scatter_probe")
    return int(issued.value)


def knn_in_clusters(X, cluster_of, n_clusters, k, device=0, stream=None, return_stats=False):
    """nomad_knn_in_clusters: the k nearest other points of every point inside its own cluster (int32 [n, k], -1 where
    the cluster is too small).  X and cluster_of: both torch tensors on the device, or both host arrays / CPU tensors;
    the result lives where the inputs live."""
    lib = load_library()
    n, d = int(X.shape[0]), int(X.shape[1])
    px, m0, keep_x = _marshal(X, np.float32, n * d)
    pc, m1, keep_c = _marshal(cluster_of, np.int32, n)
    if m0 != m1:
        raise ValueError("X and cluster_of must live in the same memory space")
    if m0 == NOMAD_DEVICE:
        import torch
        out = torch.empty((n, int(k)), dtype=torch.int32, device=keep_x.device)
        po = C.c_void_p(out.data_ptr())
        if stream is None:
            stream = torch.cuda.current_stream(device).cuda_stream
    else:
        out = np.empty((n, int(k)), dtype=np.int32)
        po = out.ctypes.data_as(C.c_void_p)
    stats = np.zeros(2, dtype=np.int64)
    rc = lib.nomad_knn_in_clusters(px, n, d, pc, int(n_clusters), int(k), po, m0, int(device), C.c_void_p(int(stream) if stream else None),
                                   stats.ctypes.data_as(C.c_void_p))
    if rc:
        raise NomadError(rc, "nomad_knn_in_clusters")
    return (out, dict(fallback_queries=int(stats[0]), filter_pairs=int(stats[1]))) if return_stats else out


def kmeans_lloyd(X, centroids, max_iters, device=0, stream=None):
    """nomad_kmeans_lloyd: Lloyd's iterations from the given centroids.  X and centroids: both torch tensors on the
    device, or both host arrays.  Returns (centroids [K, d] float32, labels [n] int32, iterations, inertia), the arrays
    where the inputs live; the input centroids are not modified."""
    lib = load_library()
    n, d = int(X.shape[0]), int(X.shape[1])
    K = int(centroids.shape[0])
    px, m0, keep_x = _marshal(X, np.float32, n * d)
    if _is_torch(centroids):
        cen = centroids.to(dtype=keep_x.dtype if _is_torch(keep_x) else None).clone().contiguous()
    else:
        cen = np.array(centroids, dtype=np.float32, order="C", copy=True)
    pc, m1, keep_c = _marshal(cen, np.float32, K * d)
    if m0 != m1:
        raise ValueError("X and centroids must live in the same memory space")
    if m0 == NOMAD_DEVICE:
        import torch
        labels = torch.empty(n, dtype=torch.int32, device=keep_x.device)
        pl = C.c_void_p(labels.data_ptr())
        if stream is None:
            stream = torch.cuda.current_stream(device).cuda_stream
    else:
        labels = np.empty(n, dtype=np.int32)
        pl = labels.ctypes.data_as(C.c_void_p)
    iters, inertia = C.c_int32(0), C.c_double(0.0)
    rc = lib.nomad_kmeans_lloyd(px, n, d, K, pc, int(max_iters), pl, C.byref(iters), C.byref(inertia), m0, int(device),
                                C.c_void_p(int(stream) if stream else None))
    if rc:
        raise NomadError(rc, "nomad_kmeans_lloyd")
    return keep_c, labels, int(iters.value), float(inertia.value)


def _two_spaces(X, Y, stream, device):
    n, d, d_low = int(X.shape[0]), int(X.shape[1]), int(Y.shape[1])
    if int(Y.shape[0]) != n:
        raise ValueError("X and Y must have one row per point each")
    px, m0, keep_x = _marshal(X, np.float32, n * d)
    py, m1, keep_y = _marshal(Y, np.float32, n * d_low)
    if m0 != m1:
        raise ValueError("X and Y must live in the same memory space")
    if m0 == NOMAD_DEVICE and stream is None:
        import torch
        stream = torch.cuda.current_stream(device).cuda_stream
    return n, d, d_low, px, py, m0, C.c_void_p(int(stream) if stream else None), (keep_x, keep_y)


def neighbourhood_preservation(X, Y, k, queries=None, device=0, stream=None):
    """nomad_neighbourhood_preservation: (hits, hits / (k * queries)) for the data X [n, d] and the projection Y [n, d_low],
    both torch tensors on the device or both host arrays; queries: None (all points) or int32 point indices in the
    same memory space."""
    lib = load_library()
    n, d, d_low, px, py, mem, st, keep = _two_spaces(X, Y, stream, device)
    pq, mq, keep_q = _marshal(queries, np.int32)
    m = n if queries is None else int(keep_q.numel() if _is_torch(keep_q) else keep_q.size)
    if queries is not None and mq != mem:
        raise ValueError("queries must live where X and Y live")
    hits = C.c_int64(0)
    rc = lib.nomad_neighbourhood_preservation(px, n, d, py, d_low, int(k), pq, 0 if queries is None else m, C.byref(hits), mem,
                                              int(device), st)
    if rc:
        raise NomadError(rc, "nomad_neighbourhood_preservation")
    return int(hits.value), hits.value / (int(k) * m)


def random_triplet_accuracy(X, Y, n_triplets, seed, device=0, stream=None):
    """nomad_random_triplet_accuracy: (agreeing triplets, agreeing fraction)."""
    lib = load_library()
    n, d, d_low, px, py, mem, st, keep = _two_spaces(X, Y, stream, device)
    agree = C.c_int64(0)
    rc = lib.nomad_random_triplet_accuracy(px, n, d, py, d_low, int(n_triplets), int(seed), C.byref(agree), mem, int(device), st)
    if rc:
        raise NomadError(rc, "nomad_random_triplet_accuracy")
    return int(agree.value), (agree.value / int(n_triplets) if n_triplets else float("nan"))


def random_triplet_accuracy_noalloc(X, Y, n_triplets, seed, device=0, stream=None):
    """nomad_random_triplet_accuracy_noalloc: the same count with no device allocation; X, Y must be device tensors."""
    lib = load_library()
    n, d, d_low, px, py, mem, st, keep = _two_spaces(X, Y, stream, device)
    if mem != NOMAD_DEVICE:
        raise ValueError("the allocation-free call takes device tensors")
    agree = C.c_int64(0)
    rc = lib.nomad_random_triplet_accuracy_noalloc(px, n, d, py, d_low, int(n_triplets), int(seed), C.byref(agree), int(device), st)
    if rc:
        raise NomadError(rc, "nomad_random_triplet_accuracy_noalloc")
    return int(agree.value), (agree.value / int(n_triplets) if n_triplets else float("nan"))


def pca_init(X, std0=0.0, device=0, stream=None, return_stats=False):
    """nomad_pca_init: theta0 [n, 2] float32 where X lives (torch tensor on the device, or host array)."""
    lib = load_library()
    n, d = int(X.shape[0]), int(X.shape[1])
    px, mem, keep = _marshal(X, np.float32, n * d)
    if mem == NOMAD_DEVICE:
        import torch
        theta = torch.empty(n, 2, dtype=torch.float32, device=keep.device)
        pt = C.c_void_p(theta.data_ptr())
        if stream is None:
            stream = torch.cuda.current_stream(device).cuda_stream
    else:
        theta = np.empty((n, 2), dtype=np.float32)
        pt = theta.ctypes.data_as(C.c_void_p)
    stats = (C.c_double * 4)()
    rc = lib.nomad_pca_init(px, n, d, float(std0), pt, stats, mem, int(device), C.c_void_p(int(stream) if stream else None))
    if rc:
        raise NomadError(rc, "nomad_pca_init")
    if return_stats:
        return theta, dict(eigenvalues=(stats[0], stats[1]), residual=stats[2], iterations=int(stats[3]))
    return theta


def kmeans_lsh_init(X, K, planes, anchors=None, device=0, stream=None, return_buckets=False):
    """nomad_kmeans_lsh_init: initial centroids [K, d] from random-hyperplane hashing.  X, planes [b, d] and anchors [b]
    (int32 point indices; None: the library puts every plane through a sample median) all torch tensors on the
    device, or all host arrays."""
    lib = load_library()
    n, d = int(X.shape[0]), int(X.shape[1])
    b = int(planes.shape[0])
    px, m0, keep_x = _marshal(X, np.float32, n * d)
    pp, m1, keep_p = _marshal(planes, np.float32, b * d)
    pa, m2, keep_a = _marshal(anchors, np.int32, b)
    if anchors is None:
        m2 = m0
    if not (m0 == m1 == m2):
        raise ValueError("X, planes and anchors must live in the same memory space")
    if m0 == NOMAD_DEVICE:
        import torch
        cen = torch.empty(int(K), d, dtype=torch.float32, device=keep_x.device)
        buckets = torch.empty(n, dtype=torch.int32, device=keep_x.device)
        pc, pb = C.c_void_p(cen.data_ptr()), C.c_void_p(buckets.data_ptr())
        if stream is None:
            stream = torch.cuda.current_stream(device).cuda_stream
    else:
        cen = np.empty((int(K), d), dtype=np.float32)
        buckets = np.empty(n, dtype=np.int32)
        pc, pb = cen.ctypes.data_as(C.c_void_p), buckets.ctypes.data_as(C.c_void_p)
    rc = lib.nomad_kmeans_lsh_init(px, n, d, int(K), pp, pa, b, pc, pb, m0, int(device), C.c_void_p(int(stream) if stream else None))
    if rc:
        raise NomadError(rc, "nomad_kmeans_lsh_init")
    return (cen, buckets) if return_buckets else cen


class Nomad:
    """One libnomad context.  Method names are the C entry points without the prefix."""

    def __init__(self, n_points, n_clusters, n_neg, noise_count=0.0, n_epochs=1, lr0=1.0, seed=0,
                 scatter_mode=SCATTER_DETERMINISTIC, device=0, stream=None, pool_size=0, pool_block=0, batches_per_epoch=1,
                 sampled_far_field=False, mean_gradient=False, pool_mode=0, pool_line=0, pool_segment=0, inverse_rank_weights=False,
                 tune=None):
        """tune: {knob name: value} passed to nomad_tune before the graph is set (see TUNE)."""
        self.lib = load_library()
        if stream is None:
            import torch
            stream = torch.cuda.current_stream(device).cuda_stream
        self.cfg = NomadConfig(C.sizeof(NomadConfig), int(n_points), int(n_clusters), int(n_neg), float(noise_count),
                               int(n_epochs), float(lr0), int(seed), int(scatter_mode), int(batches_per_epoch), int(device),
                               C.c_void_p(int(stream) if stream else None), int(pool_size), int(pool_block),
                               FAR_FIELD_SAMPLED if sampled_far_field else FAR_FIELD_EXACT, int(bool(mean_gradient)),
                               int(pool_mode), int(pool_line), int(pool_segment), int(bool(inverse_rank_weights)))
        self.n, self.R, self.s = int(n_points), int(n_clusters), int(n_neg)
        self.device = int(device)
        self.ctx = C.c_void_p()
        rc = self.lib.nomad_create(C.byref(self.cfg), C.byref(self.ctx))
        if rc:
            self.ctx = C.c_void_p()
            raise NomadError(rc, "nomad_create")
        for knob, value in (tune or {}).items():
            self._check(self.lib.nomad_tune(self.ctx, TUNE[knob], int(value)))

    @classmethod
    def from_workload(cls, w, scatter_mode=SCATTER_DETERMINISTIC, device=0, **over):
        kw = dict(n_points=w.n, n_clusters=w.n_clusters, n_neg=w.n_neg, noise_count=w.noise_count,
                  n_epochs=w.n_epochs, lr0=w.lr0, seed=w.seed, scatter_mode=scatter_mode, device=device,
                  pool_size=getattr(w, "pool_size", 0), pool_block=getattr(w, "pool_block", 0),
                  batches_per_epoch=getattr(w, "batches_per_epoch", 1),
                  sampled_far_field=getattr(w, "sampled_far_field", False),
                  mean_gradient=getattr(w, "mean_gradient", False), pool_mode=getattr(w, "pool_mode", 0),
                  pool_line=getattr(w, "pool_line", 0), pool_segment=getattr(w, "pool_segment", 0),
                  inverse_rank_weights=getattr(w, "inverse_rank_weights", False))
        kw.update(over)
        nm = cls(**kw)
        nm.set_graph(w.row_ptr, w.col_idx, w.weights, w.cluster_of, w.cluster_group)
        nm.set_embedding(w.theta0)
        return nm

    def _check(self, rc):
        if rc:
            raise NomadError(rc, self.lib.nomad_last_error(self.ctx).decode())

    def close(self):
        if getattr(self, "ctx", None) and self.ctx.value:
            self.lib.nomad_destroy(self.ctx)
            self.ctx = C.c_void_p()

    __del__ = close

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    # ---- inputs
    def set_graph(self, row_ptr, col_idx, weights, cluster_of, cluster_group=None):
        rp, m0, k0 = _marshal(row_ptr, np.int32, self.n + 1)
        ci, m1, k1 = _marshal(col_idx, np.int32)
        w, m2, k2 = _marshal(weights, np.float32)
        co, m3, k3 = _marshal(cluster_of, np.int32, self.n)
        cg, m4, k4 = _marshal(cluster_group, np.int32, self.R if cluster_group is not None else None)
        mems = {m for m in (m0, m1, m2, m3, m4) if m is not None}
        if len(mems) > 1:
            raise ValueError("all graph buffers must live in the same memory space")
        self._check(self.lib.nomad_set_graph(self.ctx, rp, ci, w, co, cg, mems.pop()))

    def set_embedding(self, theta):
        p, mem, keep = _marshal(theta, np.float32, 2 * self.n)
        self._check(self.lib.nomad_set_embedding(self.ctx, p, mem))

    # ---- the path
    def epoch(self, t):
        self._check(self.lib.nomad_epoch(self.ctx, int(t)))

    def loss(self, t_sample):
        out = C.c_double(0.0)
        self._check(self.lib.nomad_loss(self.ctx, int(t_sample), C.byref(out)))
        return out.value

    # ---- outputs (numpy on the host, or a torch tensor on the device when device=True)
    def _out(self, fn, shape, np_dtype, device_out, *pre):
        if device_out:
            import torch
            tdt = {np.float32: torch.float32, np.int32: torch.int32}[np_dtype]
            t = torch.empty(shape, dtype=tdt, device=f"cuda:{self.device}")
            self._check(fn(self.ctx, *pre, C.c_void_p(t.data_ptr()), NOMAD_DEVICE))
            return t
        a = np.empty(shape, dtype=np_dtype)
        self._check(fn(self.ctx, *pre, a.ctypes.data_as(C.c_void_p), NOMAD_HOST))
        return a

    def get_embedding(self, device=False):
        return self._out(self.lib.nomad_get_embedding, (self.n, 2), np.float32, device)

    def get_gradient(self, device=False):
        return self._out(self.lib.nomad_get_gradient, (self.n, 2), np.float32, device)

    def get_negatives(self, t, e_begin=0, e_end=None, device=False):
        e_end = self.num_edges() if e_end is None else e_end
        return self._out(self.lib.nomad_get_negatives, (e_end - e_begin, self.s), np.int32, device, int(t),
                         int(e_begin), int(e_end))

    def get_means(self):
        mu = np.empty((self.R, 2), dtype=np.float32)
        counts = np.empty(self.R, dtype=np.int64)
        self._check(self.lib.nomad_get_means(self.ctx, mu.ctypes.data_as(C.c_void_p), counts.ctypes.data_as(C.c_void_p),
                                             NOMAD_HOST))
        return mu, counts

    def get_mean_field(self):
        A = np.empty(self.n, dtype=np.float32)
        B = np.empty((self.n, 2), dtype=np.float32)
        self._check(self.lib.nomad_get_mean_field(self.ctx, A.ctypes.data_as(C.c_void_p), B.ctypes.data_as(C.c_void_p),
                                                  NOMAD_HOST))
        return A, B

    def scatter_path(self):
        """nomad_scatter_path: one of the PATH_* constants."""
        return int(self.lib.nomad_scatter_path(self.ctx))

    def device_bytes(self):
        return int(self.lib.nomad_device_bytes(self.ctx))

    def note(self):
        """Text nomad_last_error holds (after set_graph: why a slower path is in use, if one is)."""
        return self.lib.nomad_last_error(self.ctx).decode()

    def num_edges(self):
        return int(self.lib.nomad_num_edges(self.ctx))

    def profile(self, enable=True):
        self._check(self.lib.nomad_profile(self.ctx, 1 if enable else 0))

    def profile_read(self):
        """-> {kernel name: (total ms, launches)}"""
        out = {}
        for kind, name in enumerate(KERNEL_NAMES):
            ms, cnt = C.c_double(0.0), C.c_int64(0)
            self._check(self.lib.nomad_profile_read(self.ctx, kind, C.byref(ms), C.byref(cnt)))
            out[name] = (ms.value, cnt.value)
        return out
