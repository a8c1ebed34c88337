"""Compile the CPU oracle (plain C, gcc) into oracle/librps_oracle.so.

Test infrastructure: the oracle is never part of the product path.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "rps_oracle.c")
LIB = os.path.join(HERE, "librps_oracle.so")


def build(force: bool = True) -> str:
    """gcc the oracle; with force=False only when the library is missing or stale."""
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
           "-Wall", "-Wextra", SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
