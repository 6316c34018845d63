"""Builds libkilonerf_hip.so (gfx950) from csrc/*.hip with hipcc, in-tree, and libkn_peaks.so (the benchmark's
micro-benchmarks of the machine's own limits; nothing in the first library uses it)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libkilonerf_hip.so")
PEAKS_LIB = os.path.join(HERE, "libkn_peaks.so")
PEAKS_SOURCE = "kn_peaks.hip"
SOURCES = ["kn_api.hip", "kn_bucket.hip", "kn_group.hip", "kn_mlp_f32.hip", "kn_mlp_mfma.hip", "kn_render.hip", "kn_reorder.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-ffp-contract=off", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-mllvm", "-amdgpu-mfma-vgpr-form=1",
         "-I", INCLUDE, "-I", CSRC]


# The matrix-core MLP kernel uses the VALU "times two" output modifier in its double-angle recurrence; the
# compiler only emits it with flushed fp32 denormals, without IEEE mode, and when signed zeros / NaNs need
# no special care.  Only that file gets these flags; the index arithmetic elsewhere stays strict.
PER_FILE_FLAGS = {"kn_mlp_mfma.hip": ["-fgpu-flush-denormals-to-zero", "-fno-signed-zeros", "-fno-honor-nans",
                                      "-mno-amdgpu-ieee"]}


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    extra = os.environ.get("KN_EXTRA_HIPCC_FLAGS", "").split() + PER_FILE_FLAGS.get(src, [])
    subprocess.run(["hipcc", *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj], check=True)
    return obj


def build(force: bool = True) -> str:
    """Compile every HIP source and link the shared library; returns its path."""
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(INCLUDE, "kilonerf.h")]
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(os.path.getmtime(d) for d in deps):
        return LIB
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES) + 1)) as ex:
        objs = list(ex.map(_compile, SOURCES + [PEAKS_SOURCE]))
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs[:-1]], check=True)
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", PEAKS_LIB, objs[-1]], check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv))
