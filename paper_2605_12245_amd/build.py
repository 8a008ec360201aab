"""Build the HIP library (gfx950) into paper_2605_12245_amd/libsoar_hip.so."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "csrc", "soar_hip.hip")
OUT = os.path.join(HERE, "libsoar_hip.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# -ffp-contract=off: the kernels state every fused multiply-add explicitly; the
# compiler must not form others.  No fast-math: IEEE division, subnormals kept.
# Packed-FP32 instructions are disabled for device code.
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off", "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"),
]


def build(verbose: bool = False, extra=()) -> str:
    cmd = [HIPCC, *FLAGS, *extra, SRC, "-o", OUT]
    if verbose:
        print(" ".join(cmd))
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    lines = [l for l in r.stdout.splitlines()
             if l.strip() and "is not a recognized feature for this target" not in l]
    if r.returncode != 0 or verbose:
        print("\n".join(lines))
    if r.returncode != 0:
        raise RuntimeError("hipcc failed")
    return OUT


if __name__ == "__main__":
    build(verbose=True, extra=sys.argv[1:])
