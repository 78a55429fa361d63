"""Compile the C oracle into ``oracle/liboracle.so`` with gcc.

TEST INFRASTRUCTURE ONLY (see the header of ``adagc_oracle.c``).  No fast-math,
no contraction: the arithmetic is the one written in the source, in double.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "adagc_oracle.c")
LIB = os.path.join(HERE, "liboracle.so")
LIB_ALL_CORES = os.path.join(HERE, "liboracle_omp.so")    # the same source with -fopenmp


def build(force=False, all_cores=False):
    out = LIB_ALL_CORES if all_cores else LIB
    if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(SRC):
        return out
    tmp = out + ".tmp.%d" % os.getpid()
    cmd = ["gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
           "-Wall", "-Wextra"] + (["-fopenmp"] if all_cores else []) + ["-o", tmp, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, out)
    return out


if __name__ == "__main__":
    print(build(force=True))
    print(build(force=True, all_cores=True))
