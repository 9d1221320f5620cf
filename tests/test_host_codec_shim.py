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
                               "-fconstexpr-ops-limit=200000000", "-pthread", SRC, "-o", LIB])
    L = ctypes.CDLL(LIB)
    L.zc_host_encode_blocks.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    L.zc_host_decode_blocks.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    L.zc_host_encode_wave.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int]
    L.zc_host_decode_wave.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int]
    L.zc_host_region_order.argtypes = [ctypes.c_size_t, ctypes.c_size_t, ctypes.c_int]
    L.zc_host_region_order.restype = ctypes.c_size_t
    L.zc_host_accumulate4_all.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    L.zc_host_accumulate4_all.restype = None
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


def _mixed_blocks():
    """Blocks that need very different numbers of coder steps side by side: edge values, constants
    (one significant coefficient through all planes), zero blocks, ramps, noise, single spikes."""
    rng = np.random.default_rng(77)
    parts = [workloads.edge_values(12)[:2048], np.repeat(workloads.gradient_iid(256), 4), np.zeros(256, np.float32),
             workloads.gradient_iid(2048), (np.arange(1024, dtype=np.float32) * np.float32(1e-3)),
             workloads.activation_gelu(2048), np.where(rng.random(1024) < 0.1, 1.0, 0.0).astype(np.float32)]
    blocks = np.concatenate(parts).astype(np.float32).reshape(-1, 4)
    return blocks[rng.permutation(len(blocks))].reshape(-1)


@pytest.mark.parametrize("rate", RATES)
def test_lockstep_lanes_match_reference(oracle, shim, rate):
    """The per-lane codec with its wavefront-wide loop decisions taken by a vote among lanes that run
    in lockstep (16 and 5 lanes): what one lane does must not depend on its neighbours' blocks."""
    x = _mixed_blocks()[: 4 * 1500]
    nb = x.size // 4
    want_c = oracle.compress(x, rate)
    want_d = oracle.decompress(want_c, x.size, rate)
    rng = np.random.default_rng(500 + rate)
    junk = rng.integers(0, 256, size=nb * (rate // 2), dtype=np.uint8)
    junk[::3] &= rng.integers(0, 256, size=junk[::3].size, dtype=np.uint8)
    with np.errstate(all="ignore"):
        want_j = oracle.decompress(junk, x.size, rate)
    for lanes in (16, 5):
        got_c = np.zeros_like(want_c)
        assert shim.zc_host_encode_wave(rate, x.ctypes.data, nb, got_c.ctypes.data, lanes) == 0
        assert np.array_equal(got_c, want_c), (rate, lanes)
        for stream, want in ((want_c, want_d), (junk, want_j)):
            got = np.zeros(x.size, dtype=np.float32)
            assert shim.zc_host_decode_wave(rate, stream.ctypes.data, nb, got.ctypes.data, lanes) == 0
            bad = np.flatnonzero((got.view(np.uint32) != want.view(np.uint32)).reshape(-1, 4).any(axis=1))
            assert bad.size == 0, (rate, lanes, bad[:5])


def test_region_order_is_a_permutation_of_the_tiles(shim):
    """The tile order of the decompress kernels: every tile exactly once, whatever the tile count and
    region size; whole groups of eight regions are reordered (indices with the same value mod 8 walk
    through regions x, x + 8, ...), the rest stays in place."""
    for lg in (0, 2, 5, 6, 8):
        for tiles in (0, 1, 7, 8 << lg, (8 << lg) - 1, (8 << lg) + 1, 3 * (8 << lg) + 5, 12288, 65536, 36621):
            got = [shim.zc_host_region_order(v, tiles, lg) for v in range(tiles)]
            assert sorted(got) == list(range(tiles)), (lg, tiles)
            bulk = (tiles >> (lg + 3)) << (lg + 3)
            assert got[bulk:] == list(range(bulk, tiles))
            if bulk:
                mine = [got[v] for v in range(3, bulk, 8)]          # what XCD 3 walks through
                assert mine == sorted(mine) and all((t >> lg) % 8 == 3 for t in mine)


def test_rate4_accumulate_forms_on_every_block(oracle, shim):
    """The fused reduce at rate 4 adds a block to the running sum through a table and a fused
    multiply-add (plain form) unless unusual4 flags the block, in which case the tile is summed
    again in the careful form.  All 65536 two-byte blocks, against decode-then-add with the
    reference decoder, for running sums of either sign, tiny, huge and infinite; the flagged blocks
    are exactly those with exponent byte 250 and more or exponent byte 0 over a nonzero payload, and
    the plain form is wrong on some of them (so the flag is needed)."""
    W0 = np.arange(65536, dtype=np.uint16)
    stream = W0.view(np.uint8)
    decoded = oracle.decompress(stream, 4 * 65536, 4).reshape(-1, 4)
    E, payload = W0 & 0xFF, W0 >> 8
    expect_flag = (E >= 250) | ((E == 0) & (payload != 0))
    flags = np.zeros(65536, dtype=np.uint8)
    got = np.zeros((65536, 4), dtype=np.float32)
    shim.zc_host_accumulate4_all(1, 0, got.ctypes.data, flags.ctypes.data)
    assert np.array_equal(flags.astype(bool), expect_flag)
    assert np.array_equal(got.view(np.uint32), decoded.view(np.uint32))
    rng = np.random.default_rng(5)
    plain_differs = 0
    with np.errstate(over="ignore", invalid="ignore"):
        for base in (0.0, -0.0, 1e-3, -1e-3, 1e-42, -3e38, 3e38, np.inf, -np.inf):
            start = (np.float32(base) * (1 + rng.random((65536, 4), dtype=np.float32))).astype(np.float32)
            want = (start + decoded).astype(np.float32)
            for form in (0, 1):
                got = start.copy()
                shim.zc_host_accumulate4_all(0, form, got.ctypes.data, flags.ctypes.data)
                same = (got.view(np.uint32) == want.view(np.uint32)) | (np.isnan(got) & np.isnan(want))
                if form == 0:
                    assert same.all(), (base, np.flatnonzero(~same.all(axis=1))[:5])
                else:
                    assert same[~expect_flag].all()
                    plain_differs += int((~same[expect_flag]).any())
    assert plain_differs > 0
