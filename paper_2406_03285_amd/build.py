"""Compile the HIP library (csrc/rb.hip and the headers it includes -> librb.so, gfx950 only) in-tree with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "csrc", "rb.hip")
INCLUDE = os.path.join(ROOT, "include")
LIB = os.path.join(HERE, "librb.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-shared", "-fPIC",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


# A caller that is not Python: a plain C program against include/rb.h and the HIP runtime API (used by a GPU test).
CLIENT_SRC = os.path.join(ROOT, "tests", "c_client", "rb_client.c")
CLIENT = os.path.join(ROOT, "tests", "c_client", "rb_client")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", os.path.join(ROCM, "bin", "hipcc"))
    cmd = [hipcc, *HIPCC_FLAGS, "-I", INCLUDE, SRC, "-o", LIB]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    if os.path.exists(CLIENT_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-Wall", "-Werror", "-D__HIP_PLATFORM_AMD__", "-I", INCLUDE, "-I", os.path.join(ROCM, "include"),
               CLIENT_SRC, "-o", CLIENT, "-L", HERE, "-lrb", "-L", os.path.join(ROCM, "lib"), "-lamdhip64",
               "-Wl,-rpath,$ORIGIN/../../paper_2406_03285_amd", "-Wl,-rpath," + os.path.join(ROCM, "lib")]
        if verbose:
            print(" ".join(cmd))
        subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
