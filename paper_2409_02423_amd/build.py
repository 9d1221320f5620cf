"""Compile the HIP library (csrc/zc_kernels.hip, csrc/zc2d_kernels.hip, csrc/zl_kernels.hip) for gfx950 into
libzc.so next to this file.  hipcc cross-compiles without a GPU."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = [os.path.join(HERE, "csrc", f) for f in ("zc_kernels.hip", "zc2d_kernels.hip", "zl_kernels.hip")]
DEPS = SOURCES + [os.path.join(HERE, "csrc", f) for f in ("zc_codec.h", "zc_half.h", "zc2d_codec.h", "zl_codec.h")] + [
                  os.path.join(HERE, "..", "include", "zc.h")]
LIB = os.path.join(HERE, "libzc.so")
STAMP = LIB + ".stamp"   # digest of what the library was built from (file times do not survive every copy)

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
    "-ffp-contract=off",                      # every fp32 operation rounds once, as written
    "-fconstexpr-steps=200000000",            # the code tables are built at compile time
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def deps_digest(extra_flags=()):
    """Digest of every source, header and compiler flag the library depends on."""
    import hashlib
    h = hashlib.sha256(" ".join(FLAGS + list(extra_flags)).encode())
    for d in DEPS:
        h.update(os.path.basename(d).encode())
        with open(d, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def is_stale():
    """True if there is no built library or it was built from other sources than the present ones."""
    if not os.path.exists(LIB) or not os.path.exists(STAMP):
        return True
    with open(STAMP) as f:
        return f.read().strip() != deps_digest()


def build(extra_flags=(), out=None):
    """Compile every source (in parallel, one hipcc each) and link them into the library."""
    from concurrent.futures import ThreadPoolExecutor
    import tempfile
    out = out or LIB
    compile_flags = [f for f in FLAGS if f != "-shared"] + list(extra_flags)
    with tempfile.TemporaryDirectory(prefix="zc_build_") as work:
        objects = [os.path.join(work, os.path.basename(src) + ".o") for src in SOURCES]

        def compile_one(pair):
            src, obj = pair
            subprocess.check_call([HIPCC] + compile_flags + ["-c", src, "-o", obj])

        with ThreadPoolExecutor(max_workers=len(SOURCES)) as pool:
            list(pool.map(compile_one, zip(SOURCES, objects)))
        tmp = out + ".tmp.%d" % os.getpid()
        subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + objects + ["-o", tmp])
    os.replace(tmp, out)
    if out == LIB:
        with open(STAMP, "w") as f:
            f.write(deps_digest(extra_flags) + "\n")
    return out


if __name__ == "__main__":
    print(build())
