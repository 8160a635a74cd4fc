"""Build paper_2205_13603_amd/libms.so (the C-ABI library of include/ms.h) with hipcc for gfx950."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libms.so")
SOURCES = ["ms_core.cpp", "ms_interp.cpp", "ms_jit.cpp", "ms_runtime.cpp", "ms_search.cpp", "ms_model.cpp"]


def build(verbose=False):
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    cmd = ["/opt/rocm/bin/hipcc", "-O2", "-std=c++17", "-fPIC", "-shared", "-x", "hip", "--offload-arch=gfx950",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
           "-I", os.path.join(os.path.dirname(HERE), "include")] + srcs + [
           "-o", LIB, "-L/opt/rocm/lib", "-lhiprtc", "-lamdhip64", "-ldl", "-lpthread", "-Wl,-rpath,/opt/rocm/lib"]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
