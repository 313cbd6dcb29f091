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


CHECK_SRC = os.path.join(HERE, "sanitize_check.c")
CHECK_BIN = os.path.join(HERE, "sanitize_check")
CHECK_FLAGS = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-ffp-contract=off",
               "-fno-fast-math", "-std=c11", "-Wall", "-Wextra"]


def build_sanitize_check() -> str:
    """Compile sanitize_check.c (which includes the oracle's source) with AddressSanitizer and
    UndefinedBehaviorSanitizer into the executable oracle/sanitize_check; host code only."""
    newest = max(os.path.getmtime(SRC), os.path.getmtime(CHECK_SRC))
    if not (os.path.exists(CHECK_BIN) and os.path.getmtime(CHECK_BIN) >= newest):
        subprocess.run(["gcc", *CHECK_FLAGS, CHECK_SRC, "-o", CHECK_BIN, "-lm"], check=True)
    return CHECK_BIN


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
