"""Build the HIP library in-tree: hipcc, gfx950 only."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libarmt_hip.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


TIMELINE_LIB = os.path.join(HERE, "libarmt_hip_timeline.so")


def build(verbose: bool = False, timeline: bool = False) -> str:
    """timeline=True builds the probe variant of the library (see timeline.py) next to the product library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = TIMELINE_LIB if timeline else LIB
    cmd = [hipcc, *HIPCC_FLAGS, *(["-DARMT_GEMM_TIMELINE"] if timeline else []), "-o", out, os.path.join(CSRC, "armt_api.hip")]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the device-only feature flag and says so: harmless
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    return out


if __name__ == "__main__":
    import sys
    print(build(verbose=True, timeline="--timeline" in sys.argv))
