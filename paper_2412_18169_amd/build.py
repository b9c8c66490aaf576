"""Build libkun.so (the C-ABI library) and kun_ceilings (a stand-alone program that measures what
the HBM and MFMA rooflines reach on the GPU at hand) in-tree with hipcc for gfx950.

    python -m paper_2412_18169_amd.build
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SOURCES = ["pool.hip", "vmm.hip", "plan.hip", "append.hip", "decode.hip", "prefill.hip"]
LIB = os.path.join(HERE, "libkun.so")
CEILINGS = os.path.join(HERE, "kun_ceilings")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-fvisibility=hidden", "-fvisibility-inlines-hidden",
]


def build(verbose: bool = True, extra=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    srcs = [os.path.join(HERE, "csrc", s) for s in SOURCES]
    cmd = [hipcc, *FLAGS, *extra, "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
           *srcs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    build_ceilings(verbose)
    return LIB


def build_ceilings(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", *FLAGS[5:10],
           os.path.join(HERE, "csrc", "ceilings.hip"), "-o", CEILINGS]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return CEILINGS


if __name__ == "__main__":
    build(extra=sys.argv[1:])
