"""The C-ABI library loads, exports every symbol include/zc.h declares, and its
host-side logic (sizes, policy, error codes) behaves as documented.  No kernel is
launched here: every call below returns before reaching the GPU."""
import ctypes
import os
import re

import pytest

from paper_2409_02423_amd import zc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "zc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(z(?:c|c2d|l)_[a-z_0-9]+)\s*\(", text))
    assert declared == set(zc.EXPORTS)
    L = ctypes.CDLL(zc.library_path()) if os.path.exists(zc.library_path()) else zc.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_sizes_and_policy():
    assert zc.zc_version() >= 100
    for rate in range(-4, 40):
        ok = rate in (4, 8, 12, 16, 20, 24, 28, 32)
        assert zc.zc_rate_supported(rate) == ok
        assert zc.zc_compressed_size(1024, rate) == (1024 * rate // 8 if ok else 0)
    assert zc.zc_compressed_size(0, 8) == 0
    assert zc.zc_compressed_size(1, 4) == 2 and zc.zc_compressed_size(5, 4) == 4
    assert zc.zc_compressed_size(7, 24) == 24
    assert zc.zc_compressed_size(1 << 28, 4) == 1 << 27
    # low rate for data-parallel gradients, high rate for the rest (Table III)
    assert zc.zc_rate_for_class(zc.ZC_DP_GRADIENT) == 8
    for c in (zc.ZC_TP_ACTIVATION, zc.ZC_PP_ACTIVATION, zc.ZC_ZERO_PARAM, zc.ZC_OPT_STATE):
        assert zc.zc_rate_for_class(c) == 16
    assert zc.zc_rate_for_class(99) == 0
    # the two hybrid schemes (Table II, Table III)
    others = (zc.ZC_TP_ACTIVATION, zc.ZC_PP_ACTIVATION, zc.ZC_ZERO_PARAM, zc.ZC_OPT_STATE)
    assert zc.zc_codec_for_class(zc.ZC_SCHEME_ZHYBRID, zc.ZC_DP_GRADIENT) == (zc.ZC_CODEC_FIXED_RATE, 8)
    assert zc.zc_codec_for_class(zc.ZC_SCHEME_MZHYBRID, zc.ZC_DP_GRADIENT) == (zc.ZC_CODEC_FIXED_RATE, 8)
    for c in others:
        assert zc.zc_codec_for_class(zc.ZC_SCHEME_ZHYBRID, c) == (zc.ZC_CODEC_FIXED_RATE, 16)
        assert zc.zc_codec_for_class(zc.ZC_SCHEME_MZHYBRID, c) == (zc.ZC_CODEC_LOSSLESS, 0)
    for bad in ((2, 0), (0, 9), (-1, 0)):
        with pytest.raises(ValueError):
            zc.zc_codec_for_class(*bad)
    assert zc.lib().zc_codec_for_class(1, 1, None) == zc.ZC_CODEC_LOSSLESS      # the rate pointer may be NULL


def test_error_strings():
    seen = set()
    for code in range(0, -10, -1):
        s = zc.zc_strerror(code)
        assert s and s != "unknown error code"
        seen.add(s)
    assert len(seen) == 10
    assert zc.zc_strerror(-99) == "unknown error code"


def test_argument_errors_come_before_any_launch():
    L = zc.lib()
    good, odd = 0x10000, 0x10004  # never dereferenced: every call fails validation first
    assert L.zc_compress(good, 16, 7, good, 100, None) == zc.ZC_ERR_RATE
    assert L.zc_compress(None, 0, 8, None, 0, None) == zc.ZC_OK          # n == 0: nothing to do
    assert L.zc_compress(None, 16, 8, good, 100, None) == zc.ZC_ERR_NULL
    assert L.zc_compress(good, 16, 8, None, 100, None) == zc.ZC_ERR_NULL
    assert L.zc_compress(odd, 16, 8, good, 100, None) == zc.ZC_ERR_ALIGN
    assert L.zc_compress(good, 16, 8, odd, 100, None) == zc.ZC_ERR_ALIGN
    assert L.zc_compress(good, 16, 8, good, 15, None) == zc.ZC_ERR_CAPACITY
    assert L.zc_compress(good, (1 << 40) + 4, 8, good, 1 << 62, None) == zc.ZC_ERR_SIZE
    assert L.zc_decompress(good, 16, 5, good, None) == zc.ZC_ERR_RATE
    assert L.zc_decompress(None, 16, 8, good, None) == zc.ZC_ERR_NULL
    assert L.zc_decompress(good, 16, 8, odd, None) == zc.ZC_ERR_ALIGN
    assert L.zc_decompress(None, 0, 8, None, None) == zc.ZC_OK
    two = (ctypes.c_void_p * 2)(good, good)
    assert L.zc_reduce_compressed(two, 0, 16, 8, good, 100, None) == zc.ZC_ERR_K
    assert L.zc_reduce_compressed(two, 17, 16, 8, good, 100, None) == zc.ZC_ERR_K
    assert L.zc_reduce_compressed(two, 2, 16, 3, good, 100, None) == zc.ZC_ERR_RATE
    assert L.zc_reduce_compressed(two, 2, 16, 8, good, 15, None) == zc.ZC_ERR_CAPACITY
    assert L.zc_reduce_compressed(None, 2, 16, 8, good, 100, None) == zc.ZC_ERR_NULL
    assert L.zc_reduce_compressed((ctypes.c_void_p * 2)(good, None), 2, 16, 8, good, 100, None) == zc.ZC_ERR_NULL
    assert L.zc_reduce_compressed((ctypes.c_void_p * 2)(good, odd), 2, 16, 8, good, 100, None) == zc.ZC_ERR_ALIGN
    assert L.zc_reduce_compressed(two, 2, 0, 8, None, 0, None) == zc.ZC_OK
    assert L.zc_reduce_mixed(two, 2, good, 16, 8, good, 15, None) == zc.ZC_ERR_CAPACITY
    assert L.zc_reduce_mixed(two, 2, odd, 16, 8, good, 100, None) == zc.ZC_ERR_ALIGN
    assert L.zc_reduce_mixed(two, 0, good, 16, 8, good, 100, None) == zc.ZC_ERR_K
    assert L.zc_reduce_mixed(two, 2, good, 16, 8, None, 100, None) == zc.ZC_ERR_NULL
    assert L.zc_reduce_mixed(two, 2, None, 0, 8, None, 0, None) == zc.ZC_OK
    assert L.zc_reduce_decompress(two, 2, good, 16, 8, None, None) == zc.ZC_ERR_NULL
    assert L.zc_reduce_decompress(two, 2, good, 16, 8, odd, None) == zc.ZC_ERR_ALIGN
    assert L.zc_reduce_decompress(two, 17, good, 16, 8, good, None) == zc.ZC_ERR_K
    assert L.zc_reduce_decompress(two, 2, good, 16, 6, good, None) == zc.ZC_ERR_RATE
    assert L.zc_reduce_decompress(two, 2, None, 0, 8, None, None) == zc.ZC_OK
    assert L.zc_compress_half(good, 0, 16, 8, good, 100, None) == zc.ZC_ERR_DTYPE
    assert L.zc_compress_half(good, 3, 16, 8, good, 100, None) == zc.ZC_ERR_DTYPE
    assert L.zc_compress_half(good, zc.ZC_BF16, 16, 8, good, 15, None) == zc.ZC_ERR_CAPACITY
    assert L.zc_compress_half(good, zc.ZC_F16, 16, 9, good, 100, None) == zc.ZC_ERR_RATE
    assert L.zc_compress_half(None, zc.ZC_F16, 16, 8, good, 100, None) == zc.ZC_ERR_NULL
    assert L.zc_compress_half(None, zc.ZC_F16, 0, 8, None, 0, None) == zc.ZC_OK
    assert L.zc_decompress_half(good, 16, 8, 0, good, None) == zc.ZC_ERR_DTYPE
    assert L.zc_decompress_half(good, 16, 8, zc.ZC_BF16, odd, None) == zc.ZC_ERR_ALIGN
    assert L.zc_decompress_half(good, 16, 8, zc.ZC_F16, None, None) == zc.ZC_ERR_NULL


def test_binding_rejects_host_tensors():
    import torch
    with pytest.raises(TypeError):
        zc.zc_compress(torch.zeros(8), 8)
    with pytest.raises(TypeError):
        zc.zc_decompress(torch.zeros(8, dtype=torch.uint8), 8, 8)


def test_2d_sizes_and_argument_errors():
    for rate in range(-2, 36):
        ok = rate in (2, 4, 8, 16)
        assert zc.zc2d_rate_supported(rate) == ok
        assert zc.zc2d_compressed_size(64, 128, rate) == (64 * 128 * rate // 8 if ok else 0)
    assert zc.zc2d_compressed_size(0, 7, 4) == 0 and zc.zc2d_compressed_size(7, 0, 4) == 0
    assert zc.zc2d_compressed_size(1, 1, 2) == 4 and zc.zc2d_compressed_size(5, 9, 4) == 2 * 3 * 8
    assert zc.zc2d_compressed_size(6144, 43690, 4) == 1536 * 10923 * 8
    L = zc.lib()
    good, odd = 0x10000, 0x10004  # never dereferenced: every call fails validation first
    assert L.zc2d_compress(good, 4, 4, 12, good, 100, None) == zc.ZC_ERR_RATE
    assert L.zc2d_compress(None, 0, 9, 4, None, 0, None) == zc.ZC_OK
    assert L.zc2d_compress(None, 9, 0, 4, None, 0, None) == zc.ZC_OK
    assert L.zc2d_compress(None, 4, 4, 4, good, 100, None) == zc.ZC_ERR_NULL
    assert L.zc2d_compress(good, 4, 4, 4, None, 100, None) == zc.ZC_ERR_NULL
    assert L.zc2d_compress(odd, 4, 4, 4, good, 100, None) == zc.ZC_ERR_ALIGN
    assert L.zc2d_compress(good, 4, 4, 4, odd, 100, None) == zc.ZC_ERR_ALIGN
    assert L.zc2d_compress(good, 1 << 21, 1 << 20, 4, good, 1 << 62, None) == zc.ZC_ERR_SIZE
    assert L.zc2d_compress(good, 5, 9, 4, good, 47, None) == zc.ZC_ERR_CAPACITY
    assert L.zc2d_decompress(good, 4, 4, 3, good, None) == zc.ZC_ERR_RATE
    assert L.zc2d_decompress(None, 0, 0, 4, None, None) == zc.ZC_OK
    assert L.zc2d_decompress(None, 4, 4, 4, good, None) == zc.ZC_ERR_NULL
    assert L.zc2d_decompress(good, 4, 4, 4, odd, None) == zc.ZC_ERR_ALIGN
    assert L.zc2d_decompress(good, 1 << 41, 1, 4, good, None) == zc.ZC_ERR_SIZE


def test_lossless_sizes_and_argument_errors():
    assert zc.zl_max_compressed_size(0) == 32
    assert zc.zl_max_compressed_size(1) == 32 + 8 + 2048 + 32768
    assert zc.zl_max_compressed_size(8192) == 32 + 8 + 2048 + 32768
    assert zc.zl_max_compressed_size(8193) == 32 + 2 * (8 + 2048 + 32768)
    assert zc.zl_max_compressed_size(1 << 28) == 32 + (1 << 15) * (8 + 2048 + 32768)
    assert zc.zl_max_compressed_size((1 << 40) + 1) == 0
    L = zc.lib()
    good, odd = 0x10000, 0x10004  # never dereferenced: every call fails validation first
    cap = zc.zl_max_compressed_size(100)
    assert L.zl_compress(good, 100, None, cap, None) == zc.ZC_ERR_NULL
    assert L.zl_compress(None, 100, good, cap, None) == zc.ZC_ERR_NULL
    assert L.zl_compress(odd, 100, good, cap, None) == zc.ZC_ERR_ALIGN
    assert L.zl_compress(good, 100, odd, cap, None) == zc.ZC_ERR_ALIGN
    assert L.zl_compress(good, 100, good, cap - 1, None) == zc.ZC_ERR_CAPACITY
    assert L.zl_compress(good, (1 << 40) + 1, good, 1 << 62, None) == zc.ZC_ERR_SIZE
    assert L.zl_decompress(None, 64, 100, good, None) == zc.ZC_ERR_NULL
    assert L.zl_decompress(good, 64, 100, None, None) == zc.ZC_ERR_NULL
    assert L.zl_decompress(good, 39, 100, good, None) == zc.ZC_ERR_CAPACITY      # header + one table entry = 40 bytes
    assert L.zl_decompress(good, 64, 100, odd, None) == zc.ZC_ERR_ALIGN
    assert L.zl_decompress(good, 32, 0, None, None) == zc.ZC_OK                  # empty message: nothing to write
    assert L.zl_stream_bytes(None, None, None) == zc.ZC_ERR_NULL


def test_no_fallback_when_the_library_is_missing(monkeypatch, tmp_path):
    """Without the built library (and without a compiler to build it) every call raises: there
    is no other path."""
    from paper_2409_02423_amd import build as b
    monkeypatch.setattr(zc, "_lib", None)
    monkeypatch.setattr(b, "LIB", str(tmp_path / "libzc_missing.so"))

    def refuse(*a, **k):
        raise RuntimeError("no compiler here")

    monkeypatch.setattr(b, "build", refuse)
    with pytest.raises(RuntimeError):
        zc.zc_version()
    with pytest.raises(RuntimeError):
        zc.zc_compressed_size(16, 4)
