"""Compile the C oracle into oracle/liborc.so with gcc (CPU only)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "flp_oracle.c")
LIB = os.path.join(HERE, "liborc.so")
LIB_F32ACC = os.path.join(HERE, "liborc_f32acc.so")     # timing variant for the benchmark's cpu_baseline leg only


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
           "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    # the same source with fp32 running sums and -O3: timed beside the parity build, never compared against
    subprocess.run(["gcc", "-O3", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-DORC_ACC_T=float", "-o", LIB_F32ACC,
                    SRC, "-lm"], check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv))
