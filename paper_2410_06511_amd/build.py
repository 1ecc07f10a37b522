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


GEMM_INST = "f8_gemm_inst.hip"   # compiled once per (format of A, format of B, layout)


def sources():
    """(source file, extra flags, object name) of every translation unit."""
    units = []
    for src in sorted(glob.glob(os.path.join(CSRC, "*.hip"))):
        name = os.path.basename(src)
        if name == GEMM_INST:
            for fa in (0, 1):
                for fb in (0, 1):
                    for layout in (0, 1, 2):
                        units.append((src, [f"-DF8_INST_FA={fa}", f"-DF8_INST_FB={fb}", f"-DF8_INST_LAYOUT={layout}"],
                                      f"f8_gemm_inst_{fa}{fb}{layout}.o"))
        else:
            units.append((src, [], name + ".o"))
    # the GEMM instances take longest: start them first
    return sorted(units, key=lambda u: os.path.basename(u[0]) != GEMM_INST)


def build(extra=(), verbose=False) -> str:
    """Compile every source to an object (in parallel: the GEMM file dominates), then link."""
    import concurrent.futures
    import tempfile
    compile_flags = [f for f in FLAGS if f != "-shared"]
    with tempfile.TemporaryDirectory(prefix="f8build_") as tmp:
        def compile_one(unit):
            src, defs, objname = unit
            obj = os.path.join(tmp, objname)
            cmd = [HIPCC] + compile_flags + list(extra) + defs + ["-c", src, "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.run(cmd, check=True)
            return obj
        with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
            objs = list(pool.map(compile_one, sources()))
        link = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB + ".tmp"] + objs
        if verbose:
            print(" ".join(link), flush=True)
        subprocess.run(link, check=True)
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    print(build(extra=sys.argv[1:], verbose=True))
