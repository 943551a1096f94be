"""The C-ABI library loads and exports every symbol the header declares (no GPU needed)."""
import ctypes as C
import os
import re

import pytest

from paper_2505_15511_amd import _build, binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if _build.is_stale():
        _build.build_library()
    return binding.load_library()


def _declared():
    text = open(os.path.join(ROOT, "include", "nomad.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(nomad_[a-z_]+)\s*\(", text)))


def test_every_declared_entry_point_is_exported(lib):
    names = _declared()
    assert {"nomad_create", "nomad_set_graph", "nomad_epoch", "nomad_loss", "nomad_get_embedding"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name
    assert set(binding.EXPORTS) == set(names)


def test_only_the_abi_is_exported():
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", _build.LIB_PATH], capture_output=True, text=True).stdout
    syms = [l.split()[-1] for l in out.splitlines() if " T " in l]
    assert syms and all(s.startswith("nomad_") for s in syms), syms


def test_config_struct_layout_matches_header():
    # uint32 | int64 | int32 int32 | float int32 | float (pad) | uint64 | int32 int32 | int32 (pad) | void* | int32 int32 | int32 int32
    assert C.sizeof(binding.NomadConfig) == 104
    assert binding.NomadConfig.seed.offset == 40 and binding.NomadConfig.stream.offset == 64
    assert binding.NomadConfig.pool_size.offset == 72 and binding.NomadConfig.pool_block.offset == 76
    assert binding.NomadConfig.far_field.offset == 80 and binding.NomadConfig.mean_gradient.offset == 84
    assert binding.NomadConfig.pool_mode.offset == 88 and binding.NomadConfig.pool_line.offset == 92
    assert binding.NomadConfig.pool_segment.offset == 96 and binding.NomadConfig.edge_weights.offset == 100


def test_argument_errors_before_any_device_work(lib):
    ctx = C.c_void_p()
    assert lib.nomad_create(None, C.byref(ctx)) == -1
    cfg = binding.NomadConfig(C.sizeof(binding.NomadConfig), 10, 2, 5, 0.0, 10, 1.0, 1, 0, 1, 0, None)
    assert lib.nomad_create(C.byref(cfg), None) == -1
    cfg.struct_size = 8
    assert lib.nomad_create(C.byref(cfg), C.byref(ctx)) == -1
    cfg.struct_size = C.sizeof(binding.NomadConfig)
    for field, bad in (("n_points", 0), ("n_clusters", 0), ("n_neg", 17), ("n_neg", -1), ("n_epochs", 0),
                       ("scatter_mode", 2), ("batches_per_epoch", 0), ("batches_per_epoch", 4097), ("lr0", float("nan")),
                       ("n_clusters", 11), ("pool_size", 4097), ("pool_size", 64), ("far_field", 2), ("far_field", -1), ("mean_gradient", 2)):
        good = getattr(cfg, field)
        setattr(cfg, field, bad)
        assert lib.nomad_create(C.byref(cfg), C.byref(ctx)) == -1, field
        setattr(cfg, field, good)
    cfg.pool_size, cfg.pool_block, cfg.far_field = 64, 1024, 1      # the sampled far field has no pooled form
    assert lib.nomad_create(C.byref(cfg), C.byref(ctx)) == -1
    cfg.pool_size, cfg.pool_block, cfg.far_field = 0, 0, 0
    cfg.mean_gradient, cfg.far_field = 1, 1                           # gradient through the means: exact far field only
    assert lib.nomad_create(C.byref(cfg), C.byref(ctx)) == -1
    cfg.far_field, cfg.batches_per_epoch = 0, 2                       # ... and one step per epoch
    assert lib.nomad_create(C.byref(cfg), C.byref(ctx)) == -1
    cfg.mean_gradient, cfg.batches_per_epoch = 0, 1
    # the pooled sampler with distinct picks: power-of-two pool, s <= lines, whole segments, one step per epoch
    for size, block, line, seg, batches, ok in ((64, 1024, 4, 64, 1, True), (48, 1024, 1, 64, 1, False), (64, 1024, 32, 64, 1, False),
                                                (64, 1024, 4, 96, 1, False), (64, 1000, 4, 64, 1, False), (64, 1024, 4, 2048, 1, False),
                                                (64, 1024, 4, 64, 2, False), (64, 1024, 0, 0, 1, True), (1, 1024, 1, 64, 1, False),
                                                (128, 1024, 8, 64, 1, True), (128, 1024, 16, 64, 1, False)):   # a line longer than the 10 points
        cfg.pool_size, cfg.pool_block, cfg.pool_mode, cfg.pool_line, cfg.pool_segment, cfg.batches_per_epoch = size, block, 1, line, seg, batches
        rc = lib.nomad_create(C.byref(cfg), C.byref(ctx))
        assert (rc == -1) == (not ok), (size, block, line, seg, batches, rc)      # accepted: 0, or -6 where no GPU is present
        if rc == 0:
            lib.nomad_destroy(ctx)
            ctx = C.c_void_p()
    cfg.pool_size, cfg.pool_block, cfg.pool_mode, cfg.pool_line, cfg.pool_segment, cfg.batches_per_epoch = 0, 0, 0, 0, 0, 1
    cfg.pool_line = 4                                                 # lines belong to the distinct picks
    assert lib.nomad_create(C.byref(cfg), C.byref(ctx)) == -1
    cfg.pool_line, cfg.edge_weights = 0, 2
    assert lib.nomad_create(C.byref(cfg), C.byref(ctx)) == -1
    cfg.edge_weights = 0
    cfg.n_points = 2 ** 31
    assert lib.nomad_create(C.byref(cfg), C.byref(ctx)) == -4
    assert not ctx.value
    # null context is rejected everywhere, destroy(NULL) is a no-op
    lib.nomad_destroy(None)
    assert lib.nomad_epoch(None, 0) == -1
    assert lib.nomad_set_graph(None, None, None, None, None, None, 0) == -1
    assert lib.nomad_num_edges(None) == 0
    assert lib.nomad_last_error(None) == b"null context"
    assert lib.nomad_tune(None, 1, 512) == -1 and lib.nomad_scatter_path(None) == 0 and lib.nomad_device_bytes(None) == 0


def test_stand_alone_entry_points_check_arguments_before_any_device_work(lib):
    import numpy as np
    x = np.zeros((8, 4), dtype=np.float32)
    lab = np.zeros(8, dtype=np.int32)
    out = np.zeros((8, 2), dtype=np.int32)
    px, pl, po = (a.ctypes.data_as(C.c_void_p) for a in (x, lab, out))
    hits = C.c_int64(0)
    st = (C.c_double * 4)()
    H = binding.NOMAD_HOST
    # null pointers, sizes out of range, an unknown memory space: NOMAD_E_INVALID_ARG (-1) without touching a device
    assert lib.nomad_knn_in_clusters(None, 8, 4, pl, 1, 2, po, H, 0, None, None) == -1
    assert lib.nomad_knn_in_clusters(px, 8, 4, pl, 1, 33, po, H, 0, None, None) == -1
    assert lib.nomad_knn_in_clusters(px, 8, 769, pl, 1, 2, po, H, 0, None, None) == -1
    assert lib.nomad_knn_in_clusters(px, 8, 4, pl, 1, 2, po, 7, 0, None, None) == -1
    assert lib.nomad_knn_in_clusters(px, 2 ** 31, 4, pl, 1, 2, po, H, 0, None, None) == -4
    assert lib.nomad_kmeans_lloyd(px, 8, 4, 9, px, 5, pl, None, None, H, 0, None) == -1           # more centroids than points
    assert lib.nomad_kmeans_lloyd(px, 8, 4, 2, px, 0, pl, None, None, H, 0, None) == -1           # no iterations
    assert lib.nomad_kmeans_lsh_init(px, 8, 4, 8, px, pl, 2, px, None, H, 0, None) == -1          # 2^2 planes' codes < 8 buckets
    assert lib.nomad_kmeans_lsh_init(px, 8, 4, 2, px, pl, 31, px, None, H, 0, None) == -1
    assert lib.nomad_neighbourhood_preservation(px, 8, 4, px, 4, 0, None, 0, C.byref(hits), H, 0, None) == -1
    assert lib.nomad_neighbourhood_preservation(px, 8, 4, px, 4, 2, None, 5, C.byref(hits), H, 0, None) == -1   # all points, yet a count
    assert lib.nomad_neighbourhood_preservation(px, 1, 4, px, 4, 2, None, 0, C.byref(hits), H, 0, None) == -1
    assert lib.nomad_random_triplet_accuracy(px, 2, 4, px, 4, 10, 0, C.byref(hits), H, 0, None) == -1
    assert lib.nomad_random_triplet_accuracy(px, 8, 4, px, 4, -1, 0, C.byref(hits), H, 0, None) == -1
    assert lib.nomad_random_triplet_accuracy(px, 8, 4, px, 4, 10, 0, None, H, 0, None) == -1
    # the documented ranges end where the launches would no longer fit: beyond them an error code, no launch
    assert lib.nomad_random_triplet_accuracy(px, 8, 4, px, 4, 2 ** 40 + 1, 0, C.byref(hits), H, 0, None) == -4
    assert lib.nomad_random_triplet_accuracy(px, 2 ** 31 - 256, 4, px, 4, 10, 0, C.byref(hits), H, 0, None) == -4
    assert lib.nomad_random_triplet_accuracy_noalloc(px, 8, 4, px, 4, 2 ** 40 + 1, 0, C.byref(hits), 0, None) == -4
    assert lib.nomad_random_triplet_accuracy_noalloc(px, 2 ** 31 - 256, 4, px, 4, 10, 0, C.byref(hits), 0, None) == -4
    assert lib.nomad_random_triplet_accuracy_noalloc(px, 2, 4, px, 4, 10, 0, C.byref(hits), 0, None) == -1
    assert lib.nomad_random_triplet_accuracy_noalloc(None, 8, 4, px, 4, 10, 0, C.byref(hits), 0, None) == -1
    assert lib.nomad_random_triplet_accuracy_noalloc(px, 8, 4, px, 4, 10, 0, None, 0, None) == -1
    assert lib.nomad_random_triplet_accuracy_noalloc(px, 8, 4, px, 4, 10, 0, C.byref(hits), -1, None) == -1
    assert lib.nomad_pca_init(px, 8, 1, 0.0, px, st, H, 0, None) == -1
    assert lib.nomad_pca_init(px, 1, 4, 0.0, px, st, H, 0, None) == -1
    assert lib.nomad_pca_init(px, 8, 4, float("nan"), px, st, H, 0, None) == -1
    assert lib.nomad_pca_init(px, 8, 4, 0.0, px, st, H, -1, None) == -1


def test_header_is_plain_c(tmp_path):
    import os
    import shutil
    import subprocess
    if not shutil.which("gcc"):
        pytest.skip("no C compiler")
    src = tmp_path / "use_header.c"
    src.write_text('#include "nomad.h"\nint main(void) { return sizeof(nomad_config) == 104 ? 0 : 1; }\n')
    exe = tmp_path / "use_header"
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I" + inc, str(src), "-o", str(exe)], check=True)
    assert subprocess.run([str(exe)]).returncode == 0


def test_missing_library_is_an_error_not_a_fallback(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(_build, "LIB_PATH", "/nonexistent/libnomad.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        binding.load_library()
