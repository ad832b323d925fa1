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


def resource_usage(defines=()):
    """Compile the device code once more with the compiler's kernel-resource-usage remarks
    and return one row per kernel: (name, VGPRs, AGPRs, SGPRs, SGPR spills, VGPR spills,
    scratch bytes per lane, occupancy in waves per SIMD).  Template arguments of
    odsgd_kernel<W, MODE, RULE> are decoded from the mangled name."""
    import re
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [hipcc, *flags, *["-D" + d for d in defines], "--cuda-device-only", "-c", SRC, "-o", os.devnull,
           "-Rpass-analysis=kernel-resource-usage"]
    text = subprocess.run(cmd, check=True, capture_output=True, text=True).stderr
    modes = {0: "od", 1: "ssgd", 2: "global", 3: "local", 4: "copy probe", 5: "global, streamed state"}
    rules = {0: "sgd", 1: "dcasgd_c", 2: "dcasgd_a", 3: "momentum"}
    rows = []
    for block in re.split(r"remark: Function Name: ", text)[1:]:
        mangled = block.split()[0]

        def field(key):
            m = re.search(re.escape(key) + r": (\S+)", block)
            return m.group(1) if m else "?"

        m = re.search(r"odsgd_kernelILi(\d+)ELi(\d+)ELi(\d+)E", mangled)
        if m:
            wt, mode, rule = (int(x) for x in m.groups())
            name = "odsgd_kernel<%s, %s, %s>" % (wt if wt else "any W", modes.get(mode, mode), rules.get(rule, rule))
        else:
            m = re.search(r"\d+(odsgd_[a-z_]+)", mangled)
            name = m.group(1) if m else mangled
        rows.append((name, field("VGPRs"), field("AGPRs"), field("TotalSGPRs"), field("SGPRs Spill"),
                     field("VGPRs Spill"), field("ScratchSize [bytes/lane]"), field("Occupancy [waves/SIMD]")))
    return cmd, rows


if __name__ == "__main__":
    if sys.argv[1:2] == ["--resource-usage"]:
        cmd, rows = resource_usage(defines=sys.argv[2:])
        print("command: " + " ".join(cmd))
        print("| kernel | VGPRs | AGPRs | SGPRs | SGPR spills | VGPR spills | scratch B/lane | waves/SIMD |")
        print("|---|---|---|---|---|---|---|---|")
        for r in rows:
            print("| " + " | ".join(r) + " |")
    else:
        print(build(force=True, defines=sys.argv[1:]))
