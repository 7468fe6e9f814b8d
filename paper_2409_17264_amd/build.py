"""Compile the HIP libraries for gfx950: csrc/medha.hip into libmedha.so (the product)
and csrc/yardstick.hip into libmedha_yardstick.so (the benchmark's yardsticks).

Run as ``python -m paper_2409_17264_amd.build``; also called by
``__graft_entry__.build()``.  hipcc cross-compiles without a GPU.
"""
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libmedha.so")
# source file -> shared library
TARGETS = {"medha.hip": LIB, "yardstick.hip": os.path.join(HERE, "libmedha_yardstick.so")}

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-inline-asm", "-fno-gpu-rdc",
]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    found = sorted(os.path.basename(p) for p in glob.glob(os.path.join(CSRC, "*.hip")))
    assert found == sorted(TARGETS), f"every .hip source needs a target: {found}"
    for src, lib in TARGETS.items():
        cmd = [hipcc] + HIPCC_FLAGS + ["-I", INCLUDE, "-I", CSRC, os.path.join(CSRC, src),
                                       "-o", lib]
        if verbose:
            print(" ".join(cmd))
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            sys.stderr.write(res.stdout + res.stderr)
            raise RuntimeError(f"hipcc failed on {src}")
        if verbose and res.stderr:
            lines = [l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l]
            sys.stderr.write("\n".join(lines) + "\n")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
