"""The per-block codec that the GPU lanes run (csrc/zc_codec.h) is also compiled
for the host and compared, block by block and bit for bit, with the reference
codec.  This checks the kernels' logic (tables, bit transposition, stream
windowing) without a GPU; the GPU parity tests check the kernels themselves."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

from paper_2409_02423_amd import workloads

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "shim", "zc_codec_host.cpp")
LIB = os.path.join(HERE, "shim", "libzc_codec_host.so")
HDR = os.path.join(HERE, "..", "paper_2409_02423_amd", "csrc", "zc_codec.h")
RATES = (4, 8, 12, 16, 20, 24, 28, 32)


@pytest.fixture(scope="module")
def shim():
    newest = max(os.path.getmtime(SRC), os.path.getmtime(HDR))
    if not os.path.exists(LIB) or os.path.getmtime(LIB) < newest:
        subprocess.check_call(["g++", "-std=c++17", "-O2", "-fwrapv", "-ffp-contract=off", "-shared", "-fPIC",
                               "-fconstexpr-ops-limit=200000000", SRC, "-o", LIB])
    L = ctypes.CDLL(LIB)
    L.zc_host_encode_blocks.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    L.zc_host_decode_blocks.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    return L


def _enc(L, x, rate):
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.zeros(x.size // 4 * (rate // 2), dtype=np.uint8)
    assert L.zc_host_encode_blocks(rate, x.ctypes.data, x.size // 4, out.ctypes.data) == 0
    return out


def _dec(L, s, nblocks, rate):
    s = np.ascontiguousarray(s, dtype=np.uint8)
    out = np.zeros(4 * nblocks, dtype=np.float32)
    assert L.zc_host_decode_blocks(rate, s.ctypes.data, nblocks, out.ctypes.data) == 0
    return out


def _inputs():
    smooth = np.cumsum(workloads.gradient_iid(4096, std=1e-4)).astype(np.float32)  # small high-order coefficients
    ramp = (np.arange(4096, dtype=np.float32) * np.float32(0.37) - 700).astype(np.float32)
    return [workloads.edge_values(11), workloads.gradient_iid(1 << 14), workloads.activation_gelu(1 << 14),
            workloads.adam_second_moments(1 << 13), workloads.gradient_lowrank(64, 128), smooth, ramp]


@pytest.mark.parametrize("rate", RATES)
def test_encode_matches_reference(oracle, shim, rate):
    for x in _inputs():
        want = oracle.compress(x, rate)
        got = _enc(shim, x, rate)
        bad = np.flatnonzero((got != want).reshape(-1, rate // 2).any(axis=1))
        assert bad.size == 0, (rate, bad[:5], x.reshape(-1, 4)[bad[:1]])


@pytest.mark.parametrize("rate", RATES)
def test_decode_matches_reference(oracle, shim, rate):
    rng = np.random.default_rng(rate)
    for x in _inputs():
        s = oracle.compress(x, rate)
        want = oracle.decompress(s, x.size, rate)
        got = _dec(shim, s, x.size // 4, rate)
        bad = np.flatnonzero((got.view(np.uint32) != want.view(np.uint32)).reshape(-1, 4).any(axis=1))
        assert bad.size == 0, (rate, bad[:5])
    # arbitrary bytes: every string decodes, and to the same values
    for trial in range(3):
        s = rng.integers(0, 256, size=8192 * (rate // 2), dtype=np.uint8)
        if trial == 1:  # long runs of zero bits, short streams
            s &= rng.integers(0, 256, size=s.size, dtype=np.uint8) & rng.integers(0, 256, size=s.size, dtype=np.uint8)
        if trial == 2:
            s |= rng.integers(0, 256, size=s.size, dtype=np.uint8)
        with np.errstate(all="ignore"):
            want = oracle.decompress(s, 4 * 8192, rate)
        got = _dec(shim, s, 8192, rate)
        bad = np.flatnonzero((got.view(np.uint32) != want.view(np.uint32)).reshape(-1, 4).any(axis=1))
        assert bad.size == 0, (rate, trial, bad[:5])
