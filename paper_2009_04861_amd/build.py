"""Compiles the HIP library for gfx950 (hipcc cross-compiles without a GPU)."""
import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(PKG, "csrc", "tm_kernels.hip")
LIB = os.path.join(PKG, "libtm_hip.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950",
    # packed fp32 instructions are not wanted on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the per-slot loops of the training kernel must unroll completely even for
    # 20 register slots, or the automata fall out of registers into scratch
    "-mllvm", "-pragma-unroll-threshold=1000000",
    "-shared", "-fPIC",
]


def build_library(verbose=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + [SRC, "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd, stderr=None if verbose else subprocess.DEVNULL)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
