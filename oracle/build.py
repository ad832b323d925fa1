"""Compile the C oracle with gcc into oracle/libodsgd_oracle.so.

The same source is compiled twice (real=float and real=double) and linked into
one shared object.  FP contraction is switched off and no -march flag is given,
so each source line is one IEEE operation (see the header of odsgd_oracle.c).
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "odsgd_oracle.c")
LIB = os.path.join(HERE, "libodsgd_oracle.so")

CFLAGS = ["-O2", "-std=c99", "-fPIC", "-ffp-contract=off", "-fno-fast-math",
          "-fno-unsafe-math-optimizations", "-Wall", "-Wextra", "-Werror"]


def build(force=False, extra_cflags=(), lib=LIB, src=SRC):
    if (not force and os.path.exists(lib)
            and os.path.getmtime(lib) >= os.path.getmtime(src)):
        return lib
    objs = []
    for real, suffix, sqrt in (("float", "f32", "sqrtf"), ("double", "f64", "sqrt")):
        obj = lib + "." + suffix + ".o"
        cmd = ["gcc", *CFLAGS, *extra_cflags, "-DODSGD_REAL=" + real,
               "-DODSGD_SUFFIX=" + suffix, "-DODSGD_SQRT=" + sqrt, "-c", src, "-o", obj]
        subprocess.run(cmd, check=True)
        objs.append(obj)
    subprocess.run(["gcc", "-shared", "-o", lib, *objs, *extra_cflags, "-lm"], check=True)
    for o in objs:
        os.remove(o)
    return lib


THREADS_SRC = os.path.join(HERE, "threads.c")
THREADS_LIB = os.path.join(HERE, "libodsgd_oracle_threads.so")


def build_threads(force=False):
    """The static multi-thread driver used by the benchmark's all-cores baseline (threads.c)."""
    if (not force and os.path.exists(THREADS_LIB)
            and os.path.getmtime(THREADS_LIB) >= os.path.getmtime(THREADS_SRC)):
        return THREADS_LIB
    subprocess.run(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-Wall", "-Wextra", "-Werror", THREADS_SRC,
                    "-o", THREADS_LIB, "-lpthread"], check=True)
    return THREADS_LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
    print(build_threads(force="--force" in sys.argv))
