"""Compile the CPU oracle (oracle/fq_oracle.c) into oracle/libfq_oracle.so with gcc.

Test infrastructure only: the GPU library neither links nor loads the result.
`-ffp-contract=off` keeps every fp32 multiply a single correctly-rounded IEEE operation
(no fused multiply-add is formed), which the quantizer's definition relies on.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "fq_oracle.c")
OUT = os.path.join(HERE, "libfq_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(OUT) and os.path.getmtime(OUT) >= os.path.getmtime(SRC):
        return OUT
    cmd = ["gcc", "-std=c11", "-O3", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-shared", "-fPIC", "-Wall", "-Wextra", "-o", OUT, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
