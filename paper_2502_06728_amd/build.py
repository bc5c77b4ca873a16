"""Builds libdetonation.so (hipcc, gfx950) next to this file.  `python -m paper_2502_06728_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
OBJ = os.path.join(_HERE, "_build")
LIB = os.path.join(_HERE, "libdetonation.so")
MEMBENCH = os.path.join(_HERE, "membench")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
    # packed-fp32 instruction selection is switched off for every kernel of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]

# one translation unit per kernel family, compiled side by side
# (the longest-compiling units first)
UNITS = [
    # a wavefront per coefficient class (chunk 96, 128, 192, 256; 64 on small shards)
    "split_compress_256.hip", "split_compress_192.hip", "split_compress_128.hip",
    "split_compress_96.hip", "split_compress_64.hip", "split_decompress.hip",
    # two lanes per chunk (chunk 96, 128, 192, 256)
    "pair_compress_256.hip", "pair_compress_192.hip", "pair_compress_128.hip",
    "pair_compress_96.hip", "pair_decompress.hip",
    # lane per chunk, top-k with fp32 values and int32 indices, by chunk size
    "tiled_topk_s96.hip", "tiled_topk_s128.hip",
    # matrix-core kernels (every other multiple of 32)
    "mfma_compress.hip", "mfma_decompress.hip",
    # lane per chunk: narrow payloads, Decoupled AdamW, Striding / Random
    "tiled_topk_packed.hip", "tiled_topk_packed_s32.hip", "tiled_topk_ternary.hip",
    "tiled_adamw.hip", "tiled_adamw_narrow.hip", "tiled_scheme.hip", "tiled_scheme_small.hip",
    "tiled_scheme_narrow_s32.hip", "tiled_scheme_narrow_s64.hip",
    "tiled_topk_s64.hip", "tiled_topk_s32.hip", "tiled_topk_s16.hip",
    # validation, dispatch, general kernels
    "detonation.hip",
]


def _run(cmd: list[str], verbose: bool) -> None:
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed:\n{res.stderr}")
    # the host pass warns that it does not know the packed-fp32 feature: harmless
    err = "\n".join(l for l in res.stderr.splitlines()
                    if "packed-fp32-ops" not in l and "loop not unrolled" not in l)
    if verbose and "warning" in err:
        print(err, file=sys.stderr)


def _includes(path: str, seen: set[str]) -> set[str]:
    """The unit and every header it includes from csrc/ or include/, transitively."""
    if path in seen or not os.path.exists(path):
        return seen
    seen.add(path)
    for line in open(path):
        line = line.strip()
        if line.startswith("#include \""):
            _includes(os.path.normpath(os.path.join(os.path.dirname(path), line.split('"')[1])), seen)
    return seen


def _stale(unit: str, obj: str) -> bool:
    if not os.path.exists(obj):
        return True
    t = os.path.getmtime(obj)
    return any(os.path.getmtime(f) > t for f in _includes(unit, set()))


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    extra = os.environ.get("DETO_EXTRA_FLAGS", "").split()
    lib = os.environ.get("DETO_BUILD_OUT", LIB)
    obj_dir = OBJ + ("_" + os.path.basename(lib) if lib != LIB else "")
    os.makedirs(obj_dir, exist_ok=True)
    objs = [os.path.join(obj_dir, u.replace(".hip", ".o")) for u in UNITS]
    jobs = [[hipcc, *HIPCC_FLAGS, *extra, "-c", "-o", o, os.path.join(CSRC, u)]
            for u, o in zip(UNITS, objs)]
    if os.environ.get("DETO_INCREMENTAL"):
        # developer convenience: keep an object that is newer than everything its unit includes
        jobs = [j for j, u, o in zip(jobs, UNITS, objs) if _stale(os.path.join(CSRC, u), o)]
    with ThreadPoolExecutor(max_workers=max(1, min(len(jobs), 8))) as pool:
        list(pool.map(lambda c: _run(c, verbose), jobs))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs], verbose)
    # the streaming micro-benchmark (HBM ceiling, counter calibration)
    if lib == LIB:
        _run([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Wno-unused-result", "-o",
              MEMBENCH, os.path.join(CSRC, "membench.hip")], verbose)
    return lib


if __name__ == "__main__":
    print(build(verbose=True))
