"""Compile the CPU oracle (oracle/fq_oracle.c) into oracle/libfq_oracle.so with gcc.

Test infrastructure: building the checker is not using it.  The flags keep the
arithmetic plain IEEE-754: no fast-math, no FMA contraction, no x87 excess
precision (x86-64 SSE2 is the default).  OpenMP only splits channels over threads (see
fqo_set_threads); it does not touch the arithmetic.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "fq_oracle.c")
LIB = os.path.join(HERE, "libfq_oracle.so")
FLAGS = ["-std=c11", "-O2", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
         "-frounding-math", "-fopenmp", "-Wall", "-Wextra"]


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.run(["gcc", *FLAGS, SRC, "-o", tmp, "-lm"], check=True)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build())
