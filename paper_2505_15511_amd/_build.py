"""Compiles libnomad.so (hand-written HIP for gfx950) next to this package."""
from __future__ import annotations

import os
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
LIB_PATH = os.environ.get("NOMAD_LIBRARY_PATH") or os.path.join(_PKG, "libnomad.so")
SOURCES = [os.path.join(_PKG, "csrc", "nomad.hip"), os.path.join(_PKG, "csrc", "knn.hip"),
           os.path.join(_PKG, "csrc", "pca.hip")]
HEADERS = [os.path.join(_PKG, "csrc", "nomad_kernels.h"), os.path.join(_PKG, "csrc", "knn_kernels.h"),
           os.path.join(_PKG, "csrc", "metrics_kernels.h"), os.path.join(_PKG, "csrc", "philox.h"),
           os.path.join(_PKG, "csrc", "pca_kernels.h"), os.path.join(_PKG, "csrc", "host_util.h"),
           os.path.join(_ROOT, "include", "nomad.h")]


def hipcc_command(out: str = LIB_PATH) -> list:
    return ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fvisibility=hidden",
            "-munsafe-fp-atomics",
            # keep the compiler from forming packed-fp32 instructions
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-I" + os.path.join(_ROOT, "include"), "-I" + os.path.join(_PKG, "csrc"), "-o", out] + SOURCES


def build_library(verbose: bool = False) -> str:
    proc = subprocess.run(hipcc_command(), capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout + proc.stderr)
    if verbose:
        print(proc.stderr)
    return LIB_PATH


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)
