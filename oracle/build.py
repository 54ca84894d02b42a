"""Compile the CPU oracle (test infrastructure) into oracle/liboracle.so with g++."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "specache_oracle.cpp")
LIB = os.path.join(HERE, "liboracle.so")


# -O1 without fast-math and with contraction off: the quantiser's binary32
# operation order is part of its definition.
FLAGS = ["-std=c++17", "-O1", "-ffp-contract=off", "-fno-fast-math"]


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["g++", *FLAGS, "-fPIC", "-shared", "-Wall", "-Wextra", "-o", LIB, SRC]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
