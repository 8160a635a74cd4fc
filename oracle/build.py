"""Compile oracle/ms_oracle.c into oracle/libms_oracle.so with gcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "ms_oracle.c")
LIB = os.path.join(HERE, "libms_oracle.so")


LIB_F32ACC = os.path.join(HERE, "libms_oracle_f32acc.so")


def build(force=True):
    """The oracle (double accumulation), and the float-accumulating build of the same file that only the benchmark's
    CPU baseline times."""
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC) and os.path.exists(LIB_F32ACC):
        return LIB
    base = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra"]
    subprocess.run(base + ["-o", LIB, SRC, "-lm"], check=True)
    subprocess.run(base + ["-DORA_ACC_T=float", "-o", LIB_F32ACC, SRC, "-lm"], check=True)
    return LIB


if __name__ == "__main__":
    print(build())
