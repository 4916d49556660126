"""Compile the HIP library for gfx950 into paper_2311_16442_amd/libmpq.so (in-tree), and the timeline build of
the same sources (phase stamps compiled in, for timeline.py) into paper_2311_16442_amd/libmpq_timeline.so."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libmpq.so")
OUT_TIMELINE = os.path.join(HERE, "libmpq_timeline.so")
SOURCES = ["mpq_pack.cpp", "mpq_kernels.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-command-line-argument",
         # the leading scalar arguments of a kernel (up to 14 dwords) are placed in registers by the loader
         "-mllvm", "-amdgpu-kernarg-preload-count=14"]


def build(verbose: bool = False, extra=(), timeline: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = OUT_TIMELINE if timeline else OUT
    cmd = [hipcc] + FLAGS + (["-DMPQ_TIMELINE"] if timeline else []) + list(extra) + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", out]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    args = [a for a in sys.argv[1:] if a != "--timeline"]
    print(build(verbose=True, extra=args, timeline="--timeline" in sys.argv[1:]))
