"""ctypes access to the lossless reference codec (oracle/zl_ref.c).  TEST INFRASTRUCTURE ONLY.

Messages are numpy arrays of 32-bit items (float32 or uint32); the codec works on their
bit patterns."""
import ctypes

import numpy as np

from . import zc_ref

_ready = False
_u32p = ctypes.POINTER(ctypes.c_uint32)

CHUNK_WORDS = 8192
GROUPS = 256
HEADER_BYTES = 32


class StreamError(ValueError):
    pass


def lib():
    global _ready
    L = zc_ref.lib()
    if not _ready:
        L.zl_ref_word_index.restype = ctypes.c_uint32
        L.zl_ref_word_index.argtypes = [ctypes.c_uint32, ctypes.c_uint32]
        for name in ("zl_ref_planes", "zl_ref_unplanes"):
            getattr(L, name).argtypes = [_u32p, _u32p]
            getattr(L, name).restype = None
        L.zl_ref_residuals.argtypes = [_u32p, _u32p]
        L.zl_ref_residuals.restype = ctypes.c_uint32
        L.zl_ref_words.argtypes = [ctypes.c_uint32, _u32p, _u32p]
        L.zl_ref_words.restype = None
        L.zl_ref_chunks.restype = ctypes.c_size_t
        L.zl_ref_chunks.argtypes = [ctypes.c_size_t]
        L.zl_ref_max_compressed_size.restype = ctypes.c_size_t
        L.zl_ref_max_compressed_size.argtypes = [ctypes.c_size_t]
        L.zl_ref_compress.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_size_t,
                                      ctypes.POINTER(ctypes.c_size_t)]
        L.zl_ref_stream_bytes.restype = ctypes.c_size_t
        L.zl_ref_stream_bytes.argtypes = [ctypes.c_void_p, ctypes.c_size_t]
        L.zl_ref_decompress.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_size_t, ctypes.c_void_p]
        L.zl_ref_compress16.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_size_t,
                                        ctypes.POINTER(ctypes.c_size_t), ctypes.c_void_p]
        L.zl_ref_decompress16.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
        _ready = True
    return L


def _words(x):
    x = np.ascontiguousarray(x)
    if x.dtype.itemsize != 4:
        raise TypeError("32-bit items expected")
    return x.reshape(-1).view(np.uint32)


def word_index(g, j):
    return int(lib().zl_ref_word_index(int(g), int(j)))


def _stage(name, v):
    a = np.ascontiguousarray(v, dtype=np.uint32)
    assert a.shape == (32,)
    out = np.zeros(32, dtype=np.uint32)
    getattr(lib(), name)(a.ctypes.data_as(_u32p), out.ctypes.data_as(_u32p))
    return out


def residuals(w):
    """(reference, residuals) of one group of 32 words."""
    a = np.ascontiguousarray(w, dtype=np.uint32)
    assert a.shape == (32,)
    r = np.zeros(32, dtype=np.uint32)
    m = lib().zl_ref_residuals(a.ctypes.data_as(_u32p), r.ctypes.data_as(_u32p))
    return int(m), r


def words(m, r):
    a = np.ascontiguousarray(r, dtype=np.uint32)
    assert a.shape == (32,)
    w = np.zeros(32, dtype=np.uint32)
    lib().zl_ref_words(int(m), a.ctypes.data_as(_u32p), w.ctypes.data_as(_u32p))
    return w


def planes(r):
    return _stage("zl_ref_planes", r)


def unplanes(p):
    return _stage("zl_ref_unplanes", p)


def max_compressed_size(n):
    return int(lib().zl_ref_max_compressed_size(int(n)))


def compress(x, guard=0):
    """Stream (uint8 array of exactly the stream's length) for a message of 32-bit items."""
    w = _words(x)
    cap = max_compressed_size(w.size)
    out = np.full(cap + guard, 0xA5, dtype=np.uint8)
    size = ctypes.c_size_t(0)
    rc = lib().zl_ref_compress(w.ctypes.data, w.size, out.ctypes.data, cap, ctypes.byref(size))
    if rc != 0:
        raise StreamError("zl_ref_compress: %d" % rc)
    assert (out[size.value:] == 0xA5).all(), "wrote past the stream's end"
    return out[: size.value].copy()


def stream_bytes(stream):
    s = np.ascontiguousarray(stream, dtype=np.uint8)
    return int(lib().zl_ref_stream_bytes(s.ctypes.data, s.size))


def decompress(stream, n, dtype=np.uint32):
    s = np.ascontiguousarray(stream, dtype=np.uint8)
    out = np.zeros(int(n), dtype=np.uint32)
    rc = lib().zl_ref_decompress(s.ctypes.data, s.size, int(n), out.ctypes.data)
    if rc != 0:
        raise StreamError("zl_ref_decompress: %d" % rc)
    return out.view(dtype)


def _halves(x):
    x = np.ascontiguousarray(x)
    if x.dtype.itemsize != 2:
        raise TypeError("16-bit items expected")
    return x.reshape(-1).view(np.uint16)


def compress16(x, guard=0):
    """Stream for a message of 16-bit items (numpy float16, or uint16 holding bf16 bits)."""
    h = _halves(x)
    cap = max_compressed_size(h.size)
    out = np.full(cap + guard, 0xA5, dtype=np.uint8)
    work = np.zeros(max(h.size, 1), dtype=np.uint32)
    size = ctypes.c_size_t(0)
    rc = lib().zl_ref_compress16(h.ctypes.data, h.size, out.ctypes.data, cap, ctypes.byref(size), work.ctypes.data)
    if rc != 0:
        raise StreamError("zl_ref_compress16: %d" % rc)
    assert (out[size.value:] == 0xA5).all(), "wrote past the stream's end"
    return out[: size.value].copy()


def decompress16(stream, n, dtype=np.uint16):
    s = np.ascontiguousarray(stream, dtype=np.uint8)
    out = np.zeros(int(n), dtype=np.uint16)
    work = np.zeros(max(int(n), 1), dtype=np.uint32)
    rc = lib().zl_ref_decompress16(s.ctypes.data, s.size, int(n), out.ctypes.data, work.ctypes.data)
    if rc != 0:
        raise StreamError("zl_ref_decompress16: %d" % rc)
    return out.view(dtype)
