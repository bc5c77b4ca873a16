"""Builds libdetonation.so (hipcc, gfx950) next to this file.  `python -m paper_2502_06728_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libdetonation.so")
MEMBENCH = os.path.join(_HERE, "membench")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall",
    # packed-fp32 instruction selection is switched off for every kernel of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def sources() -> list[str]:
    return [os.path.join(CSRC, "detonation.hip")]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    extra = os.environ.get("DETO_EXTRA_FLAGS", "").split()
    lib = os.environ.get("DETO_BUILD_OUT", LIB)
    cmd = [hipcc, *HIPCC_FLAGS, *extra, "-o", lib, *sources()]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass warns that it does not know the packed-fp32 feature: harmless
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed:\n{res.stderr}")
    if verbose and err.strip():
        print(err, file=sys.stderr)
    # the streaming micro-benchmark (HBM ceiling, counter calibration)
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-o", MEMBENCH,
           os.path.join(CSRC, "membench.hip")]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed:\n{res.stderr}")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
