"""Compile the CPU oracle (plain C) into oracle/libvqo.so.

Flags matter: -ffp-contract=off keeps every fp32 operation a separate, correctly
rounded primitive, which is what makes the oracle's quantized outputs well defined.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "vqo.c")
LIB = os.path.join(HERE, "libvqo.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
           "-fPIC", "-shared", "-Wall", "-Wextra", "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
