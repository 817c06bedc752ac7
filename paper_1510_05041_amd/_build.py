"""Build steps: the HIP library for gfx950, and the host-only test double of it.

``build_library`` cross-compiles without a GPU (hipcc targets gfx950 explicitly).  The
libraries are built in-tree and are git-ignored.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libblasx.so")
SIM_DIR = os.path.join(ROOT, "tests", "sim")
SIM_LIB_PATH = os.path.join(SIM_DIR, "libblasx_sim.so")

HOST_SOURCES = ["blasx_api.cpp", "scheduler.cpp", "alru.cpp", "tasks.cpp"]
HIP_SOURCES = ["tile_kernels.hip", "hip_backend.hip"]
HEADERS = ["tile_step.h", "backend.h", "alru.h", "tasks.h", "scheduler.h", os.path.join("..", "..", "include", "blasx.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 ALU forms are kept out of the generated code on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _newer(target, sources):
    if not os.path.exists(target):
        return False
    t = os.path.getmtime(target)
    return all(os.path.getmtime(s) <= t for s in sources)


def build_library(force=True, verbose=False):
    """hipcc -> paper_1510_05041_amd/libblasx.so (kernels + scheduler + C ABI)."""
    srcs = [os.path.join(CSRC, s) for s in HIP_SOURCES + HOST_SOURCES]
    deps = srcs + [os.path.join(CSRC, h) for h in HEADERS]
    if not force and _newer(LIB_PATH, deps):
        return LIB_PATH
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ["-shared", "-o", LIB_PATH] + srcs
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd, stdout=None if verbose else subprocess.DEVNULL, stderr=None if verbose else subprocess.DEVNULL)
    return LIB_PATH


def build_sim(force=False):
    """g++ -> tests/sim/libblasx_sim.so: the same host code over a host-only device double."""
    srcs = [os.path.join(SIM_DIR, "sim_backend.cpp")] + [os.path.join(CSRC, s) for s in HOST_SOURCES]
    deps = srcs + [os.path.join(CSRC, h) for h in HEADERS]
    if not force and _newer(SIM_LIB_PATH, deps):
        return SIM_LIB_PATH
    cmd = ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-Wall", "-o", SIM_LIB_PATH] + srcs
    subprocess.check_call(cmd)
    return SIM_LIB_PATH
