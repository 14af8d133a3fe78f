"""Builds the HIP library in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "liblowdiff.so")
SOURCES = ["ld_api.hip", "ld_config.hip", "ld_merge_sparse.hip", "ld_recover.hip", "ld_check_diff.hip", "ld_merge_sparse_adam.hip", "ld_combine_sparse.hip", "ld_dense.hip", "ld_compress.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build_library(force: bool = True, verbose: bool = False) -> str:
    """Compiles every HIP source into liblowdiff.so; returns its path."""
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    deps = srcs + [os.path.join(CSRC, "ld_common.h"), os.path.join(CSRC, "ld_sparse_common.h"),
                   os.path.join(ROOT, "include", "lowdiff.h")]
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in deps):
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + ["-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", LIB + ".tmp"] + srcs
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building liblowdiff.so")
    os.replace(LIB + ".tmp", LIB)
    return LIB
