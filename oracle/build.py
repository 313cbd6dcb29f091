"""Compile the C oracle into oracle/libw4a4_oracle.so with gcc.

Test infrastructure only: nothing in the product path imports this.
The flags keep every fp32 operation a single, separately rounded IEEE
operation (no contraction into FMA, no fast-math reassociation).
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "w4a4_oracle.c")
LIB = os.path.join(HERE, "libw4a4_oracle.so")
FLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-fno-unsafe-math-optimizations",
         "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC"]


def build(force: bool = False) -> str:
    """Build the shared object if it is missing or older than its source."""
    if (not force and os.path.exists(LIB)
            and os.path.getmtime(LIB) >= os.path.getmtime(SRC)):
        return LIB
    cmd = ["gcc", *FLAGS, SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
