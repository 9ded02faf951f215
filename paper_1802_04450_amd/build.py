"""Builds the HIP library in-tree: ``python -m paper_1802_04450_amd.build``.

hipcc cross-compiles for gfx950 without a GPU.  Packed-fp32 code generation is switched off as the
target machines require."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsceig.so")
SOURCES = ["kernels.hip", "resident.hip", "reorder.hip", "kmeans.hip", "similarity.hip", "knn.hip", "driver.hip", "sym_eig.cpp"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fopenmp", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def source_hash() -> str:
    """SHA-256 over the kernel and driver sources (file names and contents, in name order): what a profile summary
    records so that a figure taken from it can be tied to the code it was measured on."""
    import hashlib
    h = hashlib.sha256()
    for name in sorted(os.listdir(CSRC)):
        if name.endswith((".hip", ".h", ".cpp")):
            h.update(name.encode())
            with open(os.path.join(CSRC, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()


def build(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
        if src.endswith(".cpp"):   # host-only code: AVX2/FMA (every EPYC has them), OpenMP, strict IEEE
            cmd = [hipcc, "-O3", "-std=c++17", "-fPIC", "-fopenmp", "-mavx2", "-mfma", "-c",
                   os.path.join(CSRC, src), "-o", obj]
        else:
            cmd = [hipcc, *FLAGS, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        objs.append(obj)
    cmd = [hipcc, "-shared", "-fPIC", "-fopenmp", "--offload-arch=gfx950", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
