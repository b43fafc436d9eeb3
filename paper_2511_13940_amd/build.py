"""Builds libpk.so (the C-ABI library with the gfx950 kernels) in-tree with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libpk.so")
SOURCES = [os.path.join(HERE, "csrc", "pk_kernels.hip")]
HEADERS = [os.path.join(HERE, "csrc", "pk_device.h"), os.path.join(HERE, "csrc", "pk_gemm.h"),
           os.path.join(os.path.dirname(HERE), "include", "pk.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
    # packed-fp32 VALU forms are kept off for every HIP source of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def build_library(verbose=False):
    """Compile libpk.so; always recompiles.  Returns the path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + SOURCES + ["-o", LIB_PATH]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if verbose or res.returncode != 0:
        print(" ".join(cmd))
        print(res.stdout)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building libpk.so")
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
