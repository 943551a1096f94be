"""Compiles libnomad.so (hand-written HIP for gfx950) next to this package."""
from __future__ import annotations

import os
import subprocess
import tempfile

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
LIB_PATH = os.environ.get("NOMAD_LIBRARY_PATH") or os.path.join(_PKG, "libnomad.so")
SOURCES = [os.path.join(_PKG, "csrc", "nomad.hip"), os.path.join(_PKG, "csrc", "knn.hip"),
           os.path.join(_PKG, "csrc", "pca.hip"), os.path.join(_PKG, "csrc", "probes.hip")]
HEADERS = [os.path.join(_PKG, "csrc", "nomad_kernels.h"), os.path.join(_PKG, "csrc", "knn_kernels.h"),
           os.path.join(_PKG, "csrc", "metrics_kernels.h"), os.path.join(_PKG, "csrc", "philox.h"),
           os.path.join(_PKG, "csrc", "pca_kernels.h"), os.path.join(_PKG, "csrc", "host_util.h"),
           os.path.join(_PKG, "csrc", "edge_plan.h"),
           os.path.join(_ROOT, "include", "nomad.h")]


def compile_flags() -> list:
    return ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden", "-munsafe-fp-atomics",
            # keep the compiler from forming packed-fp32 instructions
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-I" + os.path.join(_ROOT, "include"), "-I" + os.path.join(_PKG, "csrc")]


def build_library(verbose: bool = False) -> str:
    """Every source to an object file (side by side: they are independent), then one link."""
    with tempfile.TemporaryDirectory(prefix="nomad_build_") as tmp:
        objects = [os.path.join(tmp, os.path.basename(src) + ".o") for src in SOURCES]
        procs = [subprocess.Popen(["hipcc"] + compile_flags() + ["-c", src, "-o", obj], stdout=subprocess.PIPE,
                                  stderr=subprocess.STDOUT, text=True) for src, obj in zip(SOURCES, objects)]
        logs = [p.communicate()[0] for p in procs]
        if any(p.returncode != 0 for p in procs):
            raise RuntimeError("hipcc failed:\n" + "\n".join(logs))
        link = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH] + objects,
                              capture_output=True, text=True)
        if link.returncode != 0:
            raise RuntimeError("link failed:\n" + link.stdout + link.stderr)
        if verbose:
            print("\n".join(logs) + link.stderr)
    return LIB_PATH


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)
