"""Build libpsx.so (the C-ABI library) in-tree with hipcc for gfx950."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpsx.so")
SOURCES = ["psx_host.cpp", "psx_cpu.cpp", "psx_kernels.hip", "psx_runtime.hip", "psx_noalloc.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                      # no fused multiply-add: results are compared bit for bit
    "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build_lib(verbose=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", LIB]
    cmd += ["-x", "hip"] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    cmd += ["-lpthread"]
    subprocess.check_call(cmd)
    return LIB


C_DRIVER_SRC = os.path.join(ROOT, "tests", "c_abi_driver.c")
C_DRIVER = os.path.join(ROOT, "tests", "c_abi_driver")


def build_c_driver(verbose=False):
    """The plain-C user of the C ABI that tests/test_gpu_c_abi.py runs: gcc, C99, linked against
    libpsx.so (found next to it through a relative run path) and the system HIP runtime."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-Werror", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(rocm, "include"), C_DRIVER_SRC, "-o", C_DRIVER,
           "-L", HERE, "-lpsx", "-L", os.path.join(rocm, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../paper_2108_05818_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return C_DRIVER


if __name__ == "__main__":
    build_lib(verbose=True)
    build_c_driver(verbose=True)
    print(LIB)
