"""The reference codecs and the host builds of the kernels' per-lane codecs, compiled with
AddressSanitizer and UndefinedBehaviorSanitizer, run over arbitrary bytes, edge values, ragged
shapes and damaged lossless streams (tests/shim/sanitize_main.cpp).  Host code only: the
GPU kernels are checked by the parity tests."""
import os
import subprocess
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]


def test_reference_and_host_codecs_under_sanitizers():
    with tempfile.TemporaryDirectory(prefix="zc_san_") as work:
        objs = []
        for name in ("zc_ref.c", "zc2d_ref.c", "zl_ref.c"):
            obj = os.path.join(work, name + ".o")
            subprocess.check_call(["gcc", "-std=c11", "-fwrapv", "-ffp-contract=off", "-Wall"] + SAN +
                                  ["-c", os.path.join(ROOT, "oracle", name), "-o", obj])
            objs.append(obj)
        for name in ("zc_codec_host.cpp", "zc2d_codec_host.cpp", "zl_codec_host.cpp", "sanitize_main.cpp"):
            obj = os.path.join(work, name + ".o")
            subprocess.check_call(["g++", "-std=c++17", "-fwrapv", "-ffp-contract=off", "-fconstexpr-ops-limit=200000000", "-pthread"] + SAN +
                                  ["-c", os.path.join(HERE, "shim", name), "-o", obj])
            objs.append(obj)
        exe = os.path.join(work, "sanitize_main")
        subprocess.check_call(["g++", "-pthread"] + SAN + objs + ["-o", exe, "-lm"])
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
        r = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
        assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
        assert "runtime error" not in r.stderr and "ERROR: AddressSanitizer" not in r.stderr, r.stderr[-4000:]
        assert "sanitize driver: ok" in r.stdout
