"""Compile the CPU oracle (test infrastructure) with gcc.

Two builds of the same sources (the 8-bit oracle and its 4-bit-code sibling, one library): a portable one and one for x86-64-v3 hosts (hardware
FMA).  Both are bit-identical in results (fmaf is correctly rounded either way); the
second is only faster.  -ffp-contract=off keeps every rounding where the source puts it.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = [os.path.join(HERE, "trim_oracle.c"), os.path.join(HERE, "trim_oracle_fs.c")]
COMMON = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
          "-shared", "-fPIC", "-Wall", "-Wextra"]


def build(verbose: bool = False) -> None:
    for name, extra in (("libtrim_oracle.so", []),
                        ("libtrim_oracle_v3.so", ["-march=x86-64-v3"])):
        cmd = COMMON + extra + ["-o", os.path.join(HERE, name)] + SRC + ["-lm"]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)


if __name__ == "__main__":
    build(verbose=True)
    sys.exit(0)
