"""Compile the CPU oracle (plain C + OpenMP) into oracle/libc2r_oracle.so.

Test infrastructure: building the checker is not using it.  `-ffp-contract=off`
keeps the compiler from fusing or re-associating anything the source does not
spell out; `-mfma` makes the explicit fused multiply-adds single instructions.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "c2r_oracle.c")
OUT = os.path.join(HERE, "libc2r_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(OUT) and os.path.getmtime(OUT) >= os.path.getmtime(SRC):
        return OUT
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-mfma", "-ffp-contract=off", "-fno-fast-math",
           "-fPIC", "-shared", "-Wall", "-Wextra", "-o", OUT, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    print(build())
    sys.exit(0)
