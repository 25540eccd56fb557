"""Compile libivfpq.so (HIP kernels for gfx950 + host code) in-tree.

    python -m paper_2301_06672_amd.build

The host half is plain C++ (g++, OpenMP for the CPU index builder); the device half is
compiled by hipcc for gfx950 only.  No GPU is needed to build.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libivfpq.so")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")
HIPCC = os.path.join(ROCM, "bin", "hipcc")

HIP_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    # packed-FP32 VALU forms are kept off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]
HOST_FLAGS = ["-O3", "-std=c++17", "-fPIC", "-fopenmp", "-mavx2", "-mfma", "-Wall"]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)


def build(verbose: bool = False, extra_hip_flags=()) -> str:
    obj_dir = os.path.join(HERE, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    host_o = os.path.join(obj_dir, "ivfpq_host.o")
    _run(["g++", *HOST_FLAGS, "-c", os.path.join(CSRC, "ivfpq_host.cpp"), "-o", host_o], verbose)
    dev_objs = []
    for name in ("ivfpq_device", "ivfpq_build"):       # search kernels; index construction kernels
        obj = os.path.join(obj_dir, name + ".o")
        _run([HIPCC, *HIP_FLAGS, *extra_hip_flags, "-c", os.path.join(CSRC, name + ".hip"), "-o", obj], verbose)
        dev_objs.append(obj)
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-o", LIB_PATH, host_o, *dev_objs, "-lgomp"], verbose)
    return LIB_PATH


if __name__ == "__main__":
    build(verbose=True, extra_hip_flags=sys.argv[1:])
