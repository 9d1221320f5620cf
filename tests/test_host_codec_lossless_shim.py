"""The per-lane pieces of the lossless codec that the GPU runs (csrc/zl_codec.h), compiled
for the host and compared group by group with the reference's stage functions."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

from paper_2409_02423_amd import workloads

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "shim", "zl_codec_host.cpp")
LIB = os.path.join(HERE, "shim", "libzl_codec_host.so")
HDR = os.path.join(HERE, "..", "paper_2409_02423_amd", "csrc", "zl_codec.h")


@pytest.fixture(scope="module")
def shim():
    newest = max(os.path.getmtime(f) for f in (SRC, HDR))
    if not os.path.exists(LIB) or os.path.getmtime(LIB) < newest:
        subprocess.check_call(["g++", "-std=c++17", "-O2", "-shared", "-fPIC", SRC, "-o", LIB])
    L = ctypes.CDLL(LIB)
    L.zl_host_to_planes.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    L.zl_host_from_planes.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    return L


def test_planes_and_words_match_reference(shim):
    from oracle import zl_ref
    rng = np.random.default_rng(11)
    parts = [workloads.edge_values(3).view(np.uint32), workloads.gradient_iid(4096).view(np.uint32),
             rng.integers(0, 1 << 32, size=4096, dtype=np.uint64).astype(np.uint32),
             (rng.integers(0, 1 << 32, size=2048, dtype=np.uint64).astype(np.uint32) & np.uint32(0xFFFF0000)),
             np.zeros(64, dtype=np.uint32), np.full(64, 0xC0490FDB, dtype=np.uint32)]
    w = np.concatenate(parts)
    w = w[: w.size // 32 * 32].reshape(-1, 32).copy()
    groups = len(w)
    refs = np.zeros(groups, dtype=np.uint32)
    maps = np.zeros(groups, dtype=np.uint32)
    planes = np.zeros_like(w)
    shim.zl_host_to_planes(w.ctypes.data, groups, refs.ctypes.data, maps.ctypes.data, planes.ctypes.data)
    for g in range(groups):
        m, r = zl_ref.residuals(w[g])
        p = zl_ref.planes(r)
        assert refs[g] == m and np.array_equal(planes[g], p), g
        assert maps[g] == sum(1 << k for k in range(32) if p[k]), g
    back = np.zeros_like(w)
    shim.zl_host_from_planes(planes.ctypes.data, refs.ctypes.data, groups, back.ctypes.data)
    assert np.array_equal(back, w)
    # planes and references that no encoder produces: same words as the reference computes
    odd = rng.integers(0, 1 << 32, size=(200, 32), dtype=np.uint64).astype(np.uint32)
    oref = rng.integers(0, 1 << 31, size=200, dtype=np.uint64).astype(np.uint32)
    shim.zl_host_from_planes(odd.ctypes.data, oref.ctypes.data, 200, back[:200].ctypes.data)
    for g in range(200):
        assert np.array_equal(back[g], zl_ref.words(int(oref[g]), zl_ref.unplanes(odd[g]))), g
