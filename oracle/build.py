"""Compile the C oracle into oracle/libmuw_oracle.so with gcc.

Test infrastructure only.  `-ffp-contract=off` keeps every multiply and add separately rounded, which
the block scores rely on (their bit patterns decide the block selection).
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "muw_oracle.c")
LIB = os.path.join(HERE, "libmuw_oracle.so")


def build(force=False):
    if (not force and os.path.exists(LIB)
            and os.path.getmtime(LIB) >= os.path.getmtime(SRC)):
        return LIB
    cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
