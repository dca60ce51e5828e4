"""Compile the CPU oracle (test infrastructure) with gcc.

Building the checker is not using it: the product path never loads this
library.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "dsq_oracle.c")
LIB = os.path.join(HERE, "libdsq_oracle.so")

# -ffp-contract=off: every binary32 operation of the quantizer is one IEEE
# operation (no fused multiply-add is formed behind the source's back).
CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared",
          "-fPIC", "-Wall", "-Wextra"]


def build_oracle(force=True):
    if not force and os.path.exists(LIB) and \
            os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call(["gcc"] + CFLAGS + ["-o", tmp, SRC, "-lm"])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_oracle())
