"""Compile the C oracle into oracle/librandline_oracle.so with gcc.

TEST INFRASTRUCTURE ONLY: the product package never imports this module.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "randline_oracle.c")
LIB = os.path.join(HERE, "librandline_oracle.so")


def build(force: bool = False) -> str:
    """Build the shared object if it is missing or older than its source."""
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIB, SRC]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
