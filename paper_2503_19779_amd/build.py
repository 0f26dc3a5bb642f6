"""Build libpygraph_hip.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import hashlib
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = [os.path.join(HERE, "csrc", "kernels.hip"), os.path.join(HERE, "csrc", "chain.hip")]
HEADERS = [os.path.join(HERE, "csrc", "kernels.h"), os.path.join(HERE, "..", "include", "pygraph_hip.h"),
           os.path.join(HERE, "..", "include", "pygraph_hip_bench.h")]
LIB = os.path.join(HERE, "libpygraph_hip.so")
STAMP = os.path.join(HERE, "libpygraph_hip.srchash")   # hash of what LIB was built from

# -ffp-contract=off: fused multiply-adds only where the source writes them, so that every variant of a
# kernel rounds identically.  The packed-fp32 target feature is switched off for the device pass.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wextra", "-Wno-unused-parameter", "-Wno-unused-command-line-argument"]


def source_hash() -> str:
    """Hash of the sources, headers and flags: file times do not survive a copy of the tree, contents do."""
    h = hashlib.sha256(" ".join(FLAGS).encode())
    for f in SOURCES + HEADERS:
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def is_stale() -> bool:
    """True if the library is missing or was built from other sources than the ones in the tree."""
    if not os.path.exists(LIB) or not os.path.exists(STAMP):
        return True
    with open(STAMP) as fh:
        return fh.read().strip() != source_hash()


def build_library(force: bool = True, verbose: bool = False) -> str:
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + ["-o", LIB] + SOURCES
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the device-only target feature and says so; everything else is shown
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{err}")
    if verbose and err.strip():
        print(err)
    with open(STAMP, "w") as fh:
        fh.write(source_hash() + "\n")
    return LIB


if __name__ == "__main__":
    print(build_library(force=True, verbose=True))
