"""Compile the HIP sources in csrc/ into libmlora_w4.so next to this file (gfx950 only).

Every source is compiled in two passes: the device pass (gfx950 code object, with the packed
fp32 VALU forms switched off: a feature only the device target knows) and the host pass, which
embeds that code object.  The objects are then linked into one shared library.
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmlora_w4.so")

COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC"]
# packed fp32 VALU forms are kept out of the generated device code
DEVICE_ONLY = ["--cuda-device-only", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError(f"{cmd[0]} failed ({proc.returncode}):\n{proc.stderr}")
    if verbose and proc.stderr.strip():
        print(proc.stderr, file=sys.stderr)


def _compile(src, hipcc, extra, verbose):
    stem = os.path.join(OBJ, os.path.splitext(os.path.basename(src))[0])
    _run([hipcc, *COMMON, *DEVICE_ONLY, *extra, "-c", src, "-o", stem + ".co"], verbose)
    _run([hipcc, *COMMON, "--cuda-host-only", "-Xclang", "-fcuda-include-gpubinary", "-Xclang",
          stem + ".co", *extra, "-c", src, "-o", stem + ".o"], verbose)
    return stem + ".o"


def build(verbose: bool = False, extra_flags=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=4) as pool:
        objs = list(pool.map(lambda s: _compile(s, hipcc, list(extra_flags), verbose), sources()))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
