"""Builds tests/native/abi_step: a plain C99 program that links libhgca.so, the HIP runtime and the C oracle.
Run by __graft_entry__.build(); the GPU test test_gpu_native_abi.py runs the program it leaves here."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
PKG = os.path.join(ROOT, "paper_2507_03153_amd")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")
EXE = os.path.join(HERE, "abi_step")


def build(verbose: bool = False) -> str:
    cmd = ["gcc", "-std=c99", "-O2", "-Wall", "-Wextra", "-fopenmp", "-D__HIP_PLATFORM_AMD__",
           "-I" + os.path.join(ROCM, "include"), "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(ROOT, "oracle"),
           os.path.join(HERE, "abi_step.c"), os.path.join(ROOT, "oracle", "hgca_oracle.c"), "-o", EXE,
           "-L" + PKG, "-lhgca", "-Wl,-rpath,$ORIGIN/../../paper_2507_03153_amd",
           "-L" + os.path.join(ROCM, "lib"), "-lamdhip64", "-Wl,-rpath," + os.path.join(ROCM, "lib"), "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return EXE


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
