"""Compile the HIP sources in csrc/ into paper_2512_20017_amd/libpbdr.so for gfx950 (cross-compiles without a GPU)."""
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpbdr.so")

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-munsafe-fp-atomics",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function"]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(verbose: bool = False, extra=()) -> str:
    cmd = ["hipcc", *FLAGS, *extra, "-o", LIB, *sources()]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


def build_ubench(verbose: bool = False) -> str:
    """The instruction-issue micro-benchmark behind the ALU roofline figures: a stand-alone program, not part of the
    library and not built by build(); bench.py builds it on demand (python paper_2512_20017_amd/build.py --ubench)."""
    src = os.path.join(HERE, "ubench", "valu_issue.hip")
    exe = os.path.join(HERE, "ubench", "valu_issue.bin")
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-o", exe, src]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return exe


if __name__ == "__main__":
    if "--ubench" in sys.argv[1:]:
        print(build_ubench(verbose=True))
    else:
        print(build(verbose=True, extra=sys.argv[1:]))
