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


C_LAUNCH_SRC = os.path.join(os.path.dirname(HERE), "tests", "c_abi_launch.c")
C_LAUNCH_LIB = os.path.join(os.path.dirname(HERE), "tests", "libc_abi_launch.so")


def build_c_launch_check():
    """Compile the plain-C caller of the library (tests/c_abi_launch.c) with gcc as a shared object that the GPU tests
    load: it sees include/pk.h and the HIP runtime's C interface only."""
    gcc = os.environ.get("CC", "gcc")
    cmd = [gcc, "-std=c99", "-O1", "-Wall", "-Werror", "-shared", "-fPIC", "-I", os.path.join(os.path.dirname(HERE), "include"),
           "-I", "/opt/rocm/include", C_LAUNCH_SRC, "-L", HERE, "-l:libpk.so", "-L/opt/rocm/lib", "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../paper_2511_13940_amd", "-Wl,-rpath,/opt/rocm/lib", "-o", C_LAUNCH_LIB]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        print(" ".join(cmd))
        print(res.stdout)
        raise RuntimeError("gcc failed building tests/libc_abi_launch.so")
    return C_LAUNCH_LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_c_launch_check())
