"""Compile the HIP sources under csrc/ into libmka.so and the measurement micro-benchmarks under
measure/ into measure/libmka_measure.so (gfx950 only), in-tree."""
from __future__ import annotations

import concurrent.futures
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJDIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmka.so")
MEASURE_SRC = os.path.join(HERE, "measure")
MEASURE_LIB = os.path.join(MEASURE_SRC, "libmka_measure.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-f32 VALU forms are kept off for every device translation unit
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall",
         "-Wno-unused-function", "-Wno-unknown-warning-option"]


def _compile(src: str) -> str:
    obj = os.path.join(OBJDIR, os.path.basename(src) + ".o")
    cmd = [HIPCC, *FLAGS, *os.environ.get("MKA_EXTRA_HIPCC_FLAGS", "").split(), "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines()
                    if "packed-fp32-ops' is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build_library(verbose: bool = True) -> str:
    """Always recompiles every translation unit and relinks."""
    os.makedirs(OBJDIR, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    msrcs = sorted(glob.glob(os.path.join(MEASURE_SRC, "*.hip")))
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(srcs) + len(msrcs))) as ex:
        allobjs = list(ex.map(_compile, srcs + msrcs))
    objs, mobjs = allobjs[:len(srcs)], allobjs[len(srcs):]
    for lib, o in ((LIB, objs), (MEASURE_LIB, mobjs)):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *o]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print(f"built {LIB} from {len(srcs)} sources, {MEASURE_LIB} from {len(msrcs)}")
    return LIB


if __name__ == "__main__":
    build_library()
