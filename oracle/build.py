"""Compile the C oracle into oracle/libadahop_oracle.so (gcc, no GPU involved).

TEST INFRASTRUCTURE: the oracle is only ever loaded by tests, the smoke check and the benchmark's
CPU-baseline leg.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "adahop_oracle.c")
LIB = os.path.join(HERE, "libadahop_oracle.so")


def build(force: bool = False) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-Wall", "-Wextra", "-shared", "-fPIC",
           SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
