"""Compile the reference codecs (oracle/zc_ref.c, oracle/zc2d_ref.c, oracle/zl_ref.c) into oracle/libzc_ref.so.

Test infrastructure: the product library never links or loads this.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "zc_ref.c")
SOURCES = [SRC, os.path.join(HERE, "zc2d_ref.c"), os.path.join(HERE, "zl_ref.c")]
LIB = os.path.join(HERE, "libzc_ref.so")

# -fwrapv: 32-bit wrap-around is part of the format definition.
# -ffp-contract=off / no fast-math: every fp32 operation rounds once, as written.
CFLAGS = ["-O2", "-std=c11", "-fwrapv", "-ffp-contract=off", "-fno-fast-math",
          "-Wall", "-Wextra", "-shared", "-fPIC"]


def build(force=True):
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(f) for f in SOURCES):
        return LIB
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call(["gcc"] + CFLAGS + SOURCES + ["-o", tmp, "-lm"])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build())
