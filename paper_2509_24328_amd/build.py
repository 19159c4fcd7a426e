"""Build the HIP library for gfx950 in-tree: paper_2509_24328_amd/libsv.so."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsv.so")
SOURCES = ["api.hip", "row_stats.hip", "accept_estimate.hip", "select_length.hip", "verify_sample.hip",
           "profile.hip", "warp.hip", "sparse.hip", "penalty.hip"]
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
         # products are fused only where the code says fmaf: the online
         # accumulator relies on c(m) being the same rounded fp32 number
         # everywhere it is used
         "-ffp-contract=off",
         # packed-fp32 code generation is switched off on this target
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose=False):
    """Compile every HIP source into libsv.so (always recompiles)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + ["-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
