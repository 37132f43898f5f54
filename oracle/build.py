"""Compile the CPU oracle (oracle/grass_ref.c) into oracle/libgrass_ref.so with gcc.

Test infrastructure only: nothing in the product path imports this module.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "grass_ref.c")
LIB = os.path.join(HERE, "libgrass_ref.so")


def build(force: bool = False) -> str:
    """Build the shared library if it is missing or older than its source."""
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
