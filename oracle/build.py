"""Compile the CPU oracle (plain C, fp64, OpenMP) into oracle/librn50_oracle.so.

Test infrastructure: used by the tests, the smoke check and the cpu_baseline leg of
the benchmark only.  Usage: python -m oracle.build
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "rn50_oracle.c")
LIB = os.path.join(HERE, "librn50_oracle.so")


def build(force=False):
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
           "-o", LIB, SRC, "-lm"]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
