"""ctypes access to the reference CPU codec (oracle/zc_ref.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  The product package never imports this module.
All arrays are host numpy arrays.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None

_u8p = ctypes.POINTER(ctypes.c_uint8)
_f32p = ctypes.POINTER(ctypes.c_float)
_i32p = ctypes.POINTER(ctypes.c_int32)
_u32p = ctypes.POINTER(ctypes.c_uint32)


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        L.zc_ref_rate_supported.argtypes = [ctypes.c_int]
        L.zc_ref_compressed_size.restype = ctypes.c_size_t
        L.zc_ref_compressed_size.argtypes = [ctypes.c_size_t, ctypes.c_int]
        L.zc_ref_block_exponent.argtypes = [_f32p]
        L.zc_ref_quantise.argtypes = [_f32p, ctypes.c_int, _i32p]
        L.zc_ref_quantise.restype = None
        L.zc_ref_dequantise.argtypes = [_i32p, ctypes.c_int, _f32p]
        L.zc_ref_dequantise.restype = None
        L.zc_ref_fwd_lift.argtypes = [_i32p]
        L.zc_ref_fwd_lift.restype = None
        L.zc_ref_inv_lift.argtypes = [_i32p]
        L.zc_ref_inv_lift.restype = None
        L.zc_ref_negabinary.argtypes = [ctypes.c_int32]
        L.zc_ref_negabinary.restype = ctypes.c_uint32
        L.zc_ref_inv_negabinary.argtypes = [ctypes.c_uint32]
        L.zc_ref_inv_negabinary.restype = ctypes.c_int32
        L.zc_ref_encode_planes.argtypes = [_u32p, ctypes.c_int, _u8p]
        L.zc_ref_decode_planes.argtypes = [_u8p, ctypes.c_int, _u32p]
        L.zc_ref_decode_planes.restype = None
        L.zc_ref_encode_block.argtypes = [_f32p, ctypes.c_int, _u8p]
        L.zc_ref_encode_block.restype = None
        L.zc_ref_decode_block.argtypes = [_u8p, ctypes.c_int, _f32p]
        L.zc_ref_decode_block.restype = None
        L.zc_ref_compress.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int,
                                      ctypes.c_void_p, ctypes.c_size_t]
        L.zc_ref_decompress.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int,
                                        ctypes.c_void_p]
        L.zc_ref_reduce_compressed.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int,
                                               ctypes.c_size_t, ctypes.c_int,
                                               ctypes.c_void_p, ctypes.c_size_t]
        L.zc_ref_reduce_mixed.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_void_p,
                                          ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t]
        L.zc_ref_reduce_decompress.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_void_p,
                                               ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p]
        L.zc_ref_widen.argtypes = [ctypes.c_uint16, ctypes.c_int]
        L.zc_ref_widen.restype = ctypes.c_float
        L.zc_ref_narrow.argtypes = [ctypes.c_float, ctypes.c_int]
        L.zc_ref_narrow.restype = ctypes.c_uint16
        L.zc_ref_compress_half.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t, ctypes.c_int,
                                           ctypes.c_void_p, ctypes.c_size_t]
        L.zc_ref_decompress_half.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_int,
                                             ctypes.c_void_p]
        _lib = L
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def compressed_size(n, rate):
    return int(lib().zc_ref_compressed_size(n, rate))


def block_exponent(x4):
    x = _f32(x4)
    assert x.size == 4
    return int(lib().zc_ref_block_exponent(x.ctypes.data_as(_f32p)))


def quantise(x4, E):
    x = _f32(x4)
    q = np.zeros(4, dtype=np.int32)
    lib().zc_ref_quantise(x.ctypes.data_as(_f32p), int(E), q.ctypes.data_as(_i32p))
    return q


def dequantise(q4, E):
    q = np.ascontiguousarray(q4, dtype=np.int32)
    x = np.zeros(4, dtype=np.float32)
    lib().zc_ref_dequantise(q.ctypes.data_as(_i32p), int(E), x.ctypes.data_as(_f32p))
    return x


def fwd_lift(v4):
    v = np.array(v4, dtype=np.int32)
    lib().zc_ref_fwd_lift(v.ctypes.data_as(_i32p))
    return v


def inv_lift(v4):
    v = np.array(v4, dtype=np.int32)
    lib().zc_ref_inv_lift(v.ctypes.data_as(_i32p))
    return v


def negabinary(c):
    return int(lib().zc_ref_negabinary(int(c)))


def inv_negabinary(u):
    return int(lib().zc_ref_inv_negabinary(int(u)))


def encode_planes(u4, budget):
    """Returns (bits[budget] as uint8 0/1, number of bits written)."""
    u = np.ascontiguousarray(u4, dtype=np.uint32)
    bits = np.zeros(max(budget, 1), dtype=np.uint8)
    w = lib().zc_ref_encode_planes(u.ctypes.data_as(_u32p), int(budget), bits.ctypes.data_as(_u8p))
    return bits[:budget], int(w)


def decode_planes(bits, budget):
    b = np.zeros(max(budget, 1), dtype=np.uint8)
    b[:budget] = np.asarray(bits, dtype=np.uint8)[:budget]
    u = np.zeros(4, dtype=np.uint32)
    lib().zc_ref_decode_planes(b.ctypes.data_as(_u8p), int(budget), u.ctypes.data_as(_u32p))
    return u


def encode_block(x4, rate):
    x = _f32(x4)
    out = np.zeros(rate // 2, dtype=np.uint8)
    lib().zc_ref_encode_block(x.ctypes.data_as(_f32p), int(rate), out.ctypes.data_as(_u8p))
    return out


def decode_block(block_bytes, rate):
    b = np.ascontiguousarray(block_bytes, dtype=np.uint8)
    assert b.size == rate // 2
    x = np.zeros(4, dtype=np.float32)
    lib().zc_ref_decode_block(b.ctypes.data_as(_u8p), int(rate), x.ctypes.data_as(_f32p))
    return x


def compress(x, rate):
    x = _f32(x).reshape(-1)
    size = compressed_size(x.size, rate)
    out = np.zeros(size, dtype=np.uint8)
    rc = lib().zc_ref_compress(x.ctypes.data, x.size, int(rate), out.ctypes.data, out.size)
    if rc != 0:
        raise ValueError("zc_ref_compress failed: %d" % rc)
    return out


def decompress(stream, n, rate):
    s = np.ascontiguousarray(stream, dtype=np.uint8)
    if s.size < compressed_size(n, rate):
        raise ValueError("stream too short")
    out = np.zeros(n, dtype=np.float32)
    rc = lib().zc_ref_decompress(s.ctypes.data, int(n), int(rate), out.ctypes.data)
    if rc != 0:
        raise ValueError("zc_ref_decompress failed: %d" % rc)
    return out


def reduce_compressed(streams, n, rate):
    ss = [np.ascontiguousarray(s, dtype=np.uint8) for s in streams]
    size = compressed_size(n, rate)
    for s in ss:
        if s.size < size:
            raise ValueError("stream too short")
    k = len(ss)
    ptrs = (ctypes.c_void_p * max(k, 1))(*[s.ctypes.data for s in ss])
    out = np.zeros(size, dtype=np.uint8)
    rc = lib().zc_ref_reduce_compressed(ptrs, k, int(n), int(rate), out.ctypes.data, out.size)
    if rc != 0:
        raise ValueError("zc_ref_reduce_compressed failed: %d" % rc)
    return out


def _chunk_pointers(streams, n, rate):
    ss = [np.ascontiguousarray(s, dtype=np.uint8) for s in streams]
    size = compressed_size(n, rate)
    for s in ss:
        if s.size < size:
            raise ValueError("stream too short")
    return ss, (ctypes.c_void_p * max(len(ss), 1))(*[s.ctypes.data for s in ss])


def reduce_mixed(streams, local, n, rate):
    """compress((d_0 + ... + d_{k-1}) + local); local is a raw fp32 array or None."""
    ss, ptrs = _chunk_pointers(streams, n, rate)
    loc = None if local is None else _f32(local).reshape(-1)
    if loc is not None and loc.size < n:
        raise ValueError("local too short")
    out = np.zeros(compressed_size(n, rate), dtype=np.uint8)
    rc = lib().zc_ref_reduce_mixed(ptrs, len(ss), None if loc is None else loc.ctypes.data, int(n), int(rate),
                                   out.ctypes.data, out.size)
    if rc != 0:
        raise ValueError("zc_ref_reduce_mixed failed: %d" % rc)
    return out


def reduce_decompress(streams, local, n, rate):
    """(d_0 + ... + d_{k-1}) + local as fp32; local is a raw fp32 array or None."""
    ss, ptrs = _chunk_pointers(streams, n, rate)
    loc = None if local is None else _f32(local).reshape(-1)
    if loc is not None and loc.size < n:
        raise ValueError("local too short")
    out = np.zeros(n, dtype=np.float32)
    rc = lib().zc_ref_reduce_decompress(ptrs, len(ss), None if loc is None else loc.ctypes.data, int(n), int(rate),
                                        out.ctypes.data)
    if rc != 0:
        raise ValueError("zc_ref_reduce_decompress failed: %d" % rc)
    return out


BF16, F16 = 1, 2


def widen(h, dtype):
    return float(lib().zc_ref_widen(int(h), int(dtype)))


def narrow(f, dtype):
    return int(lib().zc_ref_narrow(float(np.float32(f)), int(dtype)))


def compress_half(bits, dtype, rate):
    """bits: uint16 array of bf16 (dtype=BF16) or fp16 (dtype=F16) bit patterns."""
    h = np.ascontiguousarray(bits, dtype=np.uint16).reshape(-1)
    out = np.zeros(compressed_size(h.size, rate), dtype=np.uint8)
    rc = lib().zc_ref_compress_half(h.ctypes.data, int(dtype), h.size, int(rate), out.ctypes.data, out.size)
    if rc != 0:
        raise ValueError("zc_ref_compress_half failed: %d" % rc)
    return out


def decompress_half(stream, n, rate, dtype):
    s = np.ascontiguousarray(stream, dtype=np.uint8)
    if s.size < compressed_size(n, rate):
        raise ValueError("stream too short")
    out = np.zeros(n, dtype=np.uint16)
    rc = lib().zc_ref_decompress_half(s.ctypes.data, int(n), int(rate), int(dtype), out.ctypes.data)
    if rc != 0:
        raise ValueError("zc_ref_decompress_half failed: %d" % rc)
    return out

