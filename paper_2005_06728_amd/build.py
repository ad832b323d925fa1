"""Compile the HIP library for gfx950 into paper_2005_06728_amd/libodsgd.so.

hipcc cross-compiles without a GPU.  Flags that matter for results:
  -ffp-contract=off                      no fused multiply-add (each operation rounds once)
  -fno-gpu-flush-denormals-to-zero       binary32 subnormals are kept
  -fhip-fp32-correctly-rounded-divide-sqrt   IEEE divide and square root
  -Xclang -target-feature -Xclang -packed-fp32-ops   no packed-fp32 instructions
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "csrc", "odsgd.hip")
LIB = os.path.join(HERE, "libodsgd.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
    "-ffp-contract=off", "-fno-gpu-flush-denormals-to-zero",
    "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    "-I", os.path.join(ROOT, "include"),
]


def build(force=True, defines=(), lib=LIB, extra=()):
    """Compile; `defines` are -D tuning overrides used for kernel sweeps."""
    deps = [SRC, os.path.join(ROOT, "include", "odsgd.h")]
    if (not force and os.path.exists(lib)
            and all(os.path.getmtime(lib) >= os.path.getmtime(d) for d in deps)):
        return lib
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *["-D" + d for d in defines], *extra, SRC, "-o", lib]
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    print(build(force=True, defines=sys.argv[1:]))
