"""Compile the CPU oracle (plain C, OpenMP) into oracle/liborcpconv.so."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "pconv_oracle.c")
SRCS = [SRC, os.path.join(HERE, "pconv_project_oracle.c")]
LIB = os.path.join(HERE, "liborcpconv.so")


def build(force: bool = False) -> str:
    if (not force and os.path.exists(LIB)
            and all(os.path.getmtime(LIB) >= os.path.getmtime(s) for s in SRCS)):
        return LIB
    cmd = ["gcc", "-O3", "-mavx2", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-shared", "-fPIC",
           "-Wall", "-Wextra", "-o", LIB, *SRCS, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
