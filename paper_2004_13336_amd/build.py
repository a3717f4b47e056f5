"""Builds libshardupdate.so for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess
from typing import List, Optional

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
INCLUDE = os.path.join(ROOT, "include")
LIB_PATH = os.path.join(PKG_DIR, "libshardupdate.so")

SOURCES = ["plan.cpp", "topology.cpp", "api.cpp", "profile.cpp", "copies.hip", "updates.hip", "rowplan.hip"]

# -ffp-contract=off: fused multiply-adds only where the source writes fmaf(), so every kernel
#   variant performs the same arithmetic per element.
# packed-fp32 ops are switched off for all device code.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
]


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: the library can only be built with the ROCm toolchain")


def build_library(out_path: str = LIB_PATH, extra_flags: Optional[List[str]] = None, verbose: bool = False) -> str:
    cmd = [hipcc_path()] + HIPCC_FLAGS + (extra_flags or []) + ["-I", INCLUDE, "-I", CSRC]
    cmd += ["-x", "hip"] + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", out_path]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or proc.returncode != 0:
        print(" ".join(cmd))
        print(proc.stdout)
        print(proc.stderr)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed building %s" % out_path)
    return out_path


if __name__ == "__main__":
    print(build_library(verbose=True))
