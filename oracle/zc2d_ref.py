"""ctypes access to the 2-D reference codec (oracle/zc2d_ref.c).  TEST INFRASTRUCTURE ONLY."""
import ctypes

import numpy as np

from . import zc_ref

_ready = False
_u8p = ctypes.POINTER(ctypes.c_uint8)
_f32p = ctypes.POINTER(ctypes.c_float)
_i32p = ctypes.POINTER(ctypes.c_int32)
_u32p = ctypes.POINTER(ctypes.c_uint32)


def lib():
    global _ready
    L = zc_ref.lib()
    if not _ready:
        L.zc2d_ref_compressed_size.restype = ctypes.c_size_t
        L.zc2d_ref_compressed_size.argtypes = [ctypes.c_size_t, ctypes.c_size_t, ctypes.c_int]
        L.zc2d_ref_order.argtypes = [_i32p]
        L.zc2d_ref_order.restype = None
        L.zc2d_ref_block_exponent.argtypes = [_f32p]
        L.zc2d_ref_quantise.argtypes = [_f32p, ctypes.c_int, _i32p]
        L.zc2d_ref_quantise.restype = None
        L.zc2d_ref_dequantise.argtypes = [_i32p, ctypes.c_int, _f32p]
        L.zc2d_ref_dequantise.restype = None
        L.zc2d_ref_fwd_transform.argtypes = [_i32p]
        L.zc2d_ref_fwd_transform.restype = None
        L.zc2d_ref_inv_transform.argtypes = [_i32p]
        L.zc2d_ref_inv_transform.restype = None
        L.zc2d_ref_encode_planes.argtypes = [_u32p, ctypes.c_int, _u8p]
        L.zc2d_ref_decode_planes.argtypes = [_u8p, ctypes.c_int, _u32p]
        L.zc2d_ref_decode_planes.restype = None
        L.zc2d_ref_encode_block.argtypes = [_f32p, ctypes.c_int, _u8p]
        L.zc2d_ref_encode_block.restype = None
        L.zc2d_ref_decode_block.argtypes = [_u8p, ctypes.c_int, _f32p]
        L.zc2d_ref_decode_block.restype = None
        L.zc2d_ref_compress.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_size_t, ctypes.c_int,
                                        ctypes.c_void_p, ctypes.c_size_t]
        L.zc2d_ref_decompress.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_size_t, ctypes.c_int,
                                          ctypes.c_void_p]
        L.zc2d_ref_reduce_compressed.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_size_t,
                                                 ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t]
        L.zc2d_ref_reduce_mixed.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t,
                                            ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t]
        L.zc2d_ref_reduce_decompress.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t,
                                                 ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p]
        L.zc2d_ref_compress_half.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t, ctypes.c_size_t, ctypes.c_int,
                                             ctypes.c_void_p, ctypes.c_size_t]
        L.zc2d_ref_decompress_half.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_size_t, ctypes.c_int, ctypes.c_int,
                                               ctypes.c_void_p]
        _ready = True
    return L


def compressed_size(rows, cols, rate):
    return int(lib().zc2d_ref_compressed_size(rows, cols, rate))


def order():
    o = np.zeros(16, dtype=np.int32)
    lib().zc2d_ref_order(o.ctypes.data_as(_i32p))
    return o


def block_exponent(x16):
    x = np.ascontiguousarray(x16, dtype=np.float32).reshape(16)
    return int(lib().zc2d_ref_block_exponent(x.ctypes.data_as(_f32p)))


def quantise(x16, E):
    x = np.ascontiguousarray(x16, dtype=np.float32).reshape(16)
    q = np.zeros(16, dtype=np.int32)
    lib().zc2d_ref_quantise(x.ctypes.data_as(_f32p), int(E), q.ctypes.data_as(_i32p))
    return q


def dequantise(q16, E):
    q = np.array(q16, dtype=np.int64).astype(np.int32).reshape(16)
    x = np.zeros(16, dtype=np.float32)
    lib().zc2d_ref_dequantise(q.ctypes.data_as(_i32p), int(E), x.ctypes.data_as(_f32p))
    return x


def fwd_transform(v16):
    v = np.array(v16, dtype=np.int32).reshape(16)
    lib().zc2d_ref_fwd_transform(v.ctypes.data_as(_i32p))
    return v


def inv_transform(v16):
    v = np.array(v16, dtype=np.int32).reshape(16)
    lib().zc2d_ref_inv_transform(v.ctypes.data_as(_i32p))
    return v


def encode_planes(u16, budget):
    u = np.ascontiguousarray(u16, dtype=np.uint32).reshape(16)
    bits = np.zeros(max(budget, 1), dtype=np.uint8)
    w = lib().zc2d_ref_encode_planes(u.ctypes.data_as(_u32p), int(budget), bits.ctypes.data_as(_u8p))
    return bits[:budget], int(w)


def decode_planes(bits, budget):
    b = np.zeros(max(budget, 1), dtype=np.uint8)
    b[:budget] = np.asarray(bits, dtype=np.uint8)[:budget]
    u = np.zeros(16, dtype=np.uint32)
    lib().zc2d_ref_decode_planes(b.ctypes.data_as(_u8p), int(budget), u.ctypes.data_as(_u32p))
    return u


def encode_block(x16, rate):
    x = np.ascontiguousarray(x16, dtype=np.float32).reshape(16)
    out = np.zeros(2 * rate, dtype=np.uint8)
    lib().zc2d_ref_encode_block(x.ctypes.data_as(_f32p), int(rate), out.ctypes.data_as(_u8p))
    return out


def decode_block(block_bytes, rate):
    b = np.ascontiguousarray(block_bytes, dtype=np.uint8)
    assert b.size == 2 * rate
    x = np.zeros(16, dtype=np.float32)
    lib().zc2d_ref_decode_block(b.ctypes.data_as(_u8p), int(rate), x.ctypes.data_as(_f32p))
    return x


def compress(x, rate):
    x = np.ascontiguousarray(x, dtype=np.float32)
    rows, cols = x.shape
    out = np.zeros(compressed_size(rows, cols, rate), dtype=np.uint8)
    rc = lib().zc2d_ref_compress(x.ctypes.data, rows, cols, int(rate), out.ctypes.data, out.size)
    if rc != 0:
        raise ValueError("zc2d_ref_compress failed: %d" % rc)
    return out


def decompress(stream, rows, cols, rate):
    s = np.ascontiguousarray(stream, dtype=np.uint8)
    if s.size < compressed_size(rows, cols, rate):
        raise ValueError("stream too short")
    out = np.zeros((rows, cols), dtype=np.float32)
    rc = lib().zc2d_ref_decompress(s.ctypes.data, rows, cols, int(rate), out.ctypes.data)
    if rc != 0:
        raise ValueError("zc2d_ref_decompress failed: %d" % rc)
    return out


def reduce_compressed(streams, rows, cols, rate):
    ss = [np.ascontiguousarray(s, dtype=np.uint8) for s in streams]
    size = compressed_size(rows, cols, rate)
    for s in ss:
        if s.size < size:
            raise ValueError("stream too short")
    k = len(ss)
    ptrs = (ctypes.c_void_p * max(k, 1))(*[s.ctypes.data for s in ss])
    out = np.zeros(size, dtype=np.uint8)
    rc = lib().zc2d_ref_reduce_compressed(ptrs, k, int(rows), int(cols), int(rate), out.ctypes.data, out.size)
    if rc != 0:
        raise ValueError("zc2d_ref_reduce_compressed failed: %d" % rc)
    return out


BF16, F16 = 1, 2


def compress_half(bits, dtype, rate):
    """bits: 2-D uint16 array of bf16 / fp16 bit patterns."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    rows, cols = b.shape
    out = np.zeros(compressed_size(rows, cols, rate), dtype=np.uint8)
    rc = lib().zc2d_ref_compress_half(b.ctypes.data, int(dtype), rows, cols, int(rate), out.ctypes.data, out.size)
    if rc != 0:
        raise ValueError("zc2d_ref_compress_half failed: %d" % rc)
    return out


def decompress_half(stream, rows, cols, rate, dtype):
    s = np.ascontiguousarray(stream, dtype=np.uint8)
    if s.size < compressed_size(rows, cols, rate):
        raise ValueError("stream too short")
    out = np.zeros((rows, cols), dtype=np.uint16)
    rc = lib().zc2d_ref_decompress_half(s.ctypes.data, int(rows), int(cols), int(rate), int(dtype), out.ctypes.data)
    if rc != 0:
        raise ValueError("zc2d_ref_decompress_half failed: %d" % rc)
    return out


def _pointers(streams, rows, cols, rate):
    ss = [np.ascontiguousarray(s, dtype=np.uint8) for s in streams]
    size = compressed_size(rows, cols, rate)
    for s in ss:
        if s.size < size:
            raise ValueError("stream too short")
    return ss, (ctypes.c_void_p * max(len(ss), 1))(*[s.ctypes.data for s in ss])


def _local(local, rows, cols):
    if local is None:
        return None, None
    a = np.ascontiguousarray(local, dtype=np.float32)
    assert a.shape == (rows, cols)
    return a, a.ctypes.data


def reduce_mixed(streams, local, rows, cols, rate):
    ss, ptrs = _pointers(streams, rows, cols, rate)
    keep, lp = _local(local, rows, cols)
    out = np.zeros(compressed_size(rows, cols, rate), dtype=np.uint8)
    rc = lib().zc2d_ref_reduce_mixed(ptrs, len(ss), lp, int(rows), int(cols), int(rate), out.ctypes.data, out.size)
    if rc != 0:
        raise ValueError("zc2d_ref_reduce_mixed failed: %d" % rc)
    return out


def reduce_decompress(streams, local, rows, cols, rate):
    ss, ptrs = _pointers(streams, rows, cols, rate)
    keep, lp = _local(local, rows, cols)
    out = np.zeros((rows, cols), dtype=np.float32)
    rc = lib().zc2d_ref_reduce_decompress(ptrs, len(ss), lp, int(rows), int(cols), int(rate), out.ctypes.data)
    if rc != 0:
        raise ValueError("zc2d_ref_reduce_decompress failed: %d" % rc)
    return out
