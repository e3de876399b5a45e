"""Compile the oracle's C source with gcc into oracle/liborc.so (test infrastructure).

KNNSSD_ORACLE_SRC / KNNSSD_ORACLE_LIB override the source and the output path; the mutation
test uses them to build deliberately broken copies and check that the pins notice.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.environ.get("KNNSSD_ORACLE_SRC", os.path.join(HERE, "forward.c"))
LIB = os.environ.get("KNNSSD_ORACLE_LIB", os.path.join(HERE, "liborc.so"))


def build_oracle(force: bool = False) -> str:
    if (not force) and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-mavx2", "-mfma",
           "-fno-fast-math", "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build_oracle(force=True))
