"""Build csrc/*.hip into paper_2410_06511_amd/libf8.so with hipcc for gfx950.

The library is built in-tree; nothing is installed.  `python -m
paper_2410_06511_amd.build` compiles unconditionally.
"""
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libf8.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++20", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 VALU ops
    "-ffp-contract=off",                                            # the cast's multiply must stay one rounding
    "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(extra=(), verbose=False) -> str:
    cmd = [HIPCC] + FLAGS + list(extra) + ["-o", LIB + ".tmp"] + sources()
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    print(build(extra=sys.argv[1:], verbose=True))
