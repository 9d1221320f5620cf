"""The per-block 4 x 4 codec that the GPU lanes run (csrc/zc2d_codec.h), compiled for
the host and compared block by block, bit for bit, with the 2-D reference codec."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

from paper_2409_02423_amd import workloads

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "shim", "zc2d_codec_host.cpp")
LIB = os.path.join(HERE, "shim", "libzc2d_codec_host.so")
HDRS = [os.path.join(HERE, "..", "paper_2409_02423_amd", "csrc", f) for f in ("zc2d_codec.h", "zc_codec.h")]
RATES = (2, 4, 8, 16)


@pytest.fixture(scope="module")
def shim():
    newest = max(os.path.getmtime(f) for f in [SRC] + HDRS)
    if not os.path.exists(LIB) or os.path.getmtime(LIB) < newest:
        subprocess.check_call(["g++", "-std=c++17", "-O2", "-fwrapv", "-ffp-contract=off", "-shared", "-fPIC",
                               "-fconstexpr-ops-limit=200000000", "-pthread", SRC, "-o", LIB])
    L = ctypes.CDLL(LIB)
    L.zc2d_host_encode_blocks.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    L.zc2d_host_decode_blocks.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    L.zc2d_host_wave.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int]
    return L


@pytest.fixture(scope="module")
def o2():
    from oracle import zc2d_ref
    zc2d_ref.lib()
    return zc2d_ref


def _blocks():
    smooth = np.cumsum(workloads.gradient_iid(8192, std=1e-4)).astype(np.float32)
    e = workloads.edge_values(13)
    parts = [e[: e.size // 16 * 16], workloads.gradient_iid(1 << 14), workloads.activation_gelu(1 << 14),
             workloads.adam_second_moments(1 << 12), workloads.gradient_lowrank(64, 128), smooth,
             np.repeat(workloads.parameters(256), 16), workloads.structured_blocks_4x4(3, 256).reshape(-1)]
    return np.concatenate(parts).astype(np.float32).reshape(-1, 16)


@pytest.mark.parametrize("rate", RATES)
def test_encode_and_decode_match_reference(o2, shim, rate):
    x = _blocks()
    want = np.stack([o2.encode_block(b, rate) for b in x])
    got = np.zeros_like(want)
    assert shim.zc2d_host_encode_blocks(rate, x.ctypes.data, len(x), got.ctypes.data) == 0
    bad = np.flatnonzero((got != want).any(axis=1))
    assert bad.size == 0, (rate, bad[:5], x[bad[:1]])
    wantd = np.stack([o2.decode_block(b, rate) for b in want])
    gotd = np.zeros_like(wantd)
    assert shim.zc2d_host_decode_blocks(rate, want.ctypes.data, len(x), gotd.ctypes.data) == 0
    bad = np.flatnonzero((gotd.view(np.uint32) != wantd.view(np.uint32)).any(axis=1))
    assert bad.size == 0, (rate, bad[:5])
    rng = np.random.default_rng(rate)
    for trial in range(3):   # arbitrary bytes, sparse and dense
        s = rng.integers(0, 256, size=(3000, 2 * rate), dtype=np.uint8)
        if trial == 1:
            s &= rng.integers(0, 256, size=s.shape, dtype=np.uint8) & rng.integers(0, 256, size=s.shape, dtype=np.uint8)
        if trial == 2:
            s |= rng.integers(0, 256, size=s.shape, dtype=np.uint8)
        with np.errstate(all="ignore"):
            wantd = np.stack([o2.decode_block(b, rate) for b in s])
        gotd = np.zeros_like(wantd)
        assert shim.zc2d_host_decode_blocks(rate, s.ctypes.data, len(s), gotd.ctypes.data) == 0
        bad = np.flatnonzero((gotd.view(np.uint32) != wantd.view(np.uint32)).any(axis=1))
        assert bad.size == 0, (rate, trial, bad[:5])


@pytest.mark.parametrize("rate", RATES)
def test_lockstep_lanes_match_reference(o2, shim, rate):
    """The per-lane codec with its wavefront-wide loop decisions taken by a vote among lanes that run
    in lockstep (16 and 5 lanes), on blocks that need very different numbers of steps side by side
    (shuffled), and on arbitrary bytes: what a lane decodes must not depend on its neighbours."""
    rng = np.random.default_rng(700 + rate)
    x = _blocks()
    x = np.ascontiguousarray(x[rng.permutation(len(x))[:1200]])
    want = np.stack([o2.encode_block(b, rate) for b in x])
    wantd = np.stack([o2.decode_block(b, rate) for b in want])
    junk = rng.integers(0, 256, size=(1200, 2 * rate), dtype=np.uint8)
    junk[::3] &= rng.integers(0, 256, size=junk[::3].shape, dtype=np.uint8)
    with np.errstate(all="ignore"):
        wantj = np.stack([o2.decode_block(b, rate) for b in junk])
    for lanes in (16, 5):
        got = np.zeros_like(want)
        assert shim.zc2d_host_wave(rate, 1, x.ctypes.data, len(x), got.ctypes.data, lanes) == 0
        assert np.array_equal(got, want), (rate, lanes)
        for stream, expect in ((want, wantd), (junk, wantj)):
            gotd = np.zeros_like(expect)
            assert shim.zc2d_host_wave(rate, 0, stream.ctypes.data, len(stream), gotd.ctypes.data, lanes) == 0
            bad = np.flatnonzero((gotd.view(np.uint32) != expect.view(np.uint32)).any(axis=1))
            assert bad.size == 0, (rate, lanes, bad[:5])
