"""NOMAD Projection epoch path for AMD MI355X: a C-ABI HIP library (libnomad.so) and its binding.

Importing the package loads nothing; ``binding.load_library()`` opens the shared library and
raises if it has not been built."""
from .binding import (Nomad, NomadError, NomadConfig, load_library, knn_in_clusters, kmeans_lloyd, neighbourhood_preservation,
                      random_triplet_accuracy, random_triplet_accuracy_noalloc, pca_init, kmeans_lsh_init, SCATTER_ATOMIC, SCATTER_DETERMINISTIC,
                      NOMAD_DEVICE, NOMAD_HOST, FAR_FIELD_EXACT, FAR_FIELD_SAMPLED, PATH_ATOMIC_FP32, PATH_BINNED,
                      PATH_BINNED_POOLED, PATH_FIXED_ATOMICS, PATH_NAMES, POOL_PICKS16, POOL_DISTINCT, POOL_STRATIFIED)  # noqa: F401
