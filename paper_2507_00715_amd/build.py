"""Build libearn.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libearn.so")
CALIB_LIB = os.path.join(HERE, "libearn_calib.so")   # the benchmark's calibration micro-kernels: not in libearn.so
SOURCES = ["api.hip", "compact.hip", "decode.hip", "prefill.hip", "stats.hip", "beam.hip", "linear.hip", "backward.hip"]
CALIB_SOURCES = ["calib.hip"]
# packed fp32 VALU ops are switched off for every device compilation (they have misbehaved on these machines)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src: str, extra) -> str:
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    cmd = ["hipcc", *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        print(err, file=sys.stderr)
    return obj


def build(extra_flags=(), verbose: bool = True) -> str:
    """Compile every source (always recompiles) and link libearn.so. Returns its path."""
    with concurrent.futures.ThreadPoolExecutor(max_workers=9) as ex:
        objs = list(ex.map(lambda s: _compile(s, list(extra_flags)), SOURCES + CALIB_SOURCES))
    n = len(SOURCES)
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs[:n]], check=True)
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", CALIB_LIB, *objs[n:]], check=True)
    if verbose:
        print(f"built {LIB} and {CALIB_LIB}")
    return LIB


if __name__ == "__main__":
    build(extra_flags=sys.argv[1:])
