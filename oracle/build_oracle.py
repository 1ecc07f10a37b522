"""Compile the C oracle into oracle/libf8_oracle.so with the host gcc.

Test infrastructure: the product never loads this library.
Flags: no fast-math and no FMA contraction, so every fp32 operation is the
single IEEE operation the source shows; OpenMP only parallelises over
independent output elements.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "f8_oracle.c")
LIB = os.path.join(HERE, "libf8_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC",
           "-Wall", "-Wextra", "-o", LIB + ".tmp", SRC, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    print(build())
