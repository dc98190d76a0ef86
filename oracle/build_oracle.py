"""Builds oracle/libkvco.so from oracle/kvco.c with gcc (test infrastructure only)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libkvco.so")


def build(force: bool = True) -> str:
    src = os.path.join(HERE, "kvco.c")
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(
        os.path.getmtime(src), os.path.getmtime(os.path.join(HERE, "kvco.h"))
    ):
        return LIB
    cmd = [
        "gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC", "-shared",
        "-Wall", "-Wextra", "-o", LIB, src, "-lm",
    ]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
