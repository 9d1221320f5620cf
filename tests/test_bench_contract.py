"""bench.py measures one GPU only: asking for more ends with a message, before anything touches a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)
    assert not r.stdout.strip().startswith("{")


def test_roofline_counters_come_from_the_tracked_profile():
    """bench.py takes HBM traffic and VALU instruction counts of the headline kernels from the
    rocprofv3 summary under profiles/: every kernel it names has a row there with both
    figures, the traffic is within a few percent of the algorithmic bytes, and a kernel of
    that name exists in the built library."""
    sys.path.insert(0, ROOT)
    import bench
    from paper_2409_02423_amd import build
    counters = bench.profiled_counters()
    n, rate = 1 << 28, 4
    for call, kernel in bench.KERNEL_NAMES.items():
        row = counters.get(kernel)
        assert row and "traffic_bytes" in row and "valu_wave_insts" in row, (kernel, row)
        alg = bench.algorithmic_bytes(call, n, rate, k=2)
        assert alg <= row["traffic_bytes"] <= 1.05 * alg, (kernel, row, alg)
    if os.path.exists(build.LIB):
        symbols = subprocess.run(["nm", "-C", build.LIB], capture_output=True, text=True).stdout
        for kernel in bench.KERNEL_NAMES.values():
            assert kernel in symbols, kernel
    assert bench.profiled_counters(os.path.join(ROOT, "profiles", "no_such_file.md")) == {}
