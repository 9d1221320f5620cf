"""Python binding of libzc (include/zc.h): argument marshalling only.

Every function has the name and meaning of the C entry point it calls; tensors
are torch CUDA tensors used as device memory, and the kernels are enqueued on
torch's current stream unless a stream is given.  There is no fallback: if the
HIP library cannot be loaded, every call raises.
"""
import ctypes
import os

import torch  # loads the HIP runtime that libzc.so binds to

from . import build as _build

ZC_OK = 0
ZC_ERR_NULL, ZC_ERR_RATE, ZC_ERR_SIZE, ZC_ERR_CAPACITY = -1, -2, -3, -4
ZC_ERR_K, ZC_ERR_ALIGN, ZC_ERR_LAUNCH, ZC_ERR_DTYPE, ZC_ERR_STREAM = -5, -6, -7, -8, -9
ZC_F32, ZC_BF16, ZC_F16 = 0, 1, 2
ZC_DP_GRADIENT, ZC_TP_ACTIVATION, ZC_PP_ACTIVATION, ZC_ZERO_PARAM, ZC_OPT_STATE = range(5)
ZC_SCHEME_ZHYBRID, ZC_SCHEME_MZHYBRID = 0, 1
ZC_CODEC_FIXED_RATE, ZC_CODEC_LOSSLESS = 0, 1

EXPORTS = ("zc_version", "zc_strerror", "zc_rate_supported", "zc_rate_for_class", "zc_codec_for_class", "zc_compressed_size",
           "zc_compress", "zc_decompress", "zc_reduce_compressed", "zc_reduce_mixed", "zc_reduce_decompress",
           "zc_compress_half", "zc_decompress_half",
           "zc2d_rate_supported", "zc2d_compressed_size", "zc2d_compress", "zc2d_decompress", "zc2d_reduce_compressed",
           "zc2d_compress_half", "zc2d_decompress_half", "zc2d_reduce_mixed", "zc2d_reduce_decompress",
           "zl_max_compressed_size", "zl_compress", "zl_stream_bytes", "zl_decompress", "zl_compress16", "zl_decompress16")

_lib = None


class ZcError(RuntimeError):
    def __init__(self, code, what):
        super().__init__("%s failed: %s (%d)" % (what, zc_strerror(code), code))
        self.code = code


def library_path():
    return _build.LIB


def lib():
    """The loaded C library.  Builds it first if there is none or if the one there was built
    from other sources than the present ones (so a changed kernel is never measured or tested
    through an old binary); a failed build raises."""
    global _lib
    if _lib is None:
        if _build.is_stale():
            _build.build()
        L = ctypes.CDLL(_build.LIB)
        L.zc_version.restype = ctypes.c_int
        L.zc_strerror.restype = ctypes.c_char_p
        L.zc_strerror.argtypes = [ctypes.c_int]
        L.zc_rate_supported.argtypes = [ctypes.c_int]
        L.zc_rate_for_class.argtypes = [ctypes.c_int]
        L.zc_codec_for_class.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
        L.zc_compressed_size.restype = ctypes.c_size_t
        L.zc_compressed_size.argtypes = [ctypes.c_size_t, ctypes.c_int]
        L.zc_compress.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p,
                                  ctypes.c_size_t, ctypes.c_void_p]
        L.zc_decompress.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p,
                                    ctypes.c_void_p]
        L.zc_reduce_compressed.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_size_t,
                                           ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.zc_reduce_mixed.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t,
                                      ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.zc_reduce_decompress.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_void_p,
                                           ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        L.zc_compress_half.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p,
                                       ctypes.c_size_t, ctypes.c_void_p]
        L.zc_decompress_half.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                         ctypes.c_void_p]
        L.zc2d_rate_supported.argtypes = [ctypes.c_int]
        L.zc2d_compressed_size.restype = ctypes.c_size_t
        L.zc2d_compressed_size.argtypes = [ctypes.c_size_t, ctypes.c_size_t, ctypes.c_int]
        L.zc2d_compress.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p,
                                    ctypes.c_size_t, ctypes.c_void_p]
        L.zc2d_decompress.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_size_t, ctypes.c_int,
                                      ctypes.c_void_p, ctypes.c_void_p]
        L.zc2d_compress_half.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t, ctypes.c_size_t, ctypes.c_int,
                                         ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.zc2d_decompress_half.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_size_t, ctypes.c_int, ctypes.c_int,
                                           ctypes.c_void_p, ctypes.c_void_p]
        L.zc2d_reduce_compressed.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_size_t, ctypes.c_size_t,
                                             ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.zc2d_reduce_mixed.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t,
                                        ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.zc2d_reduce_decompress.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t,
                                             ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        L.zl_max_compressed_size.restype = ctypes.c_size_t
        L.zl_max_compressed_size.argtypes = [ctypes.c_size_t]
        L.zl_compress.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.zl_stream_bytes.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_size_t), ctypes.c_void_p]
        L.zl_decompress.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
        L.zl_compress16.argtypes = L.zl_compress.argtypes
        L.zl_decompress16.argtypes = L.zl_decompress.argtypes
        _lib = L
    return _lib


def zc_version():
    return int(lib().zc_version())


def zc_strerror(code):
    return lib().zc_strerror(int(code)).decode()


def zc_rate_supported(rate):
    return bool(lib().zc_rate_supported(int(rate)))


def zc_rate_for_class(message_class):
    return int(lib().zc_rate_for_class(int(message_class)))


def zc_codec_for_class(scheme, message_class):
    """(codec, rate) for a message class under a scheme; raises for unknown ones."""
    rate = ctypes.c_int(0)
    codec = int(lib().zc_codec_for_class(int(scheme), int(message_class), ctypes.byref(rate)))
    if codec < 0:
        raise ValueError("unknown scheme or message class")
    return codec, int(rate.value)


def zc_compressed_size(n, rate):
    return int(lib().zc_compressed_size(int(n), int(rate)))


def _stream_handle(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check_device_tensor(t, dtype, what):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError("%s must be a contiguous CUDA tensor of dtype %s" % (what, dtype))


def _new_stream_buffer(n, rate, device):
    size = zc_compressed_size(n, rate)
    if size == 0 and n != 0:
        raise ZcError(ZC_ERR_RATE, "zc_compressed_size")
    return torch.empty(size, dtype=torch.uint8, device=device)


def zc_compress(d_in, rate, d_out=None, stream=None):
    """fp32 CUDA tensor -> uint8 CUDA tensor of zc_compressed_size(n, rate) bytes."""
    _check_device_tensor(d_in, torch.float32, "d_in")
    n = d_in.numel()
    if d_out is None:
        d_out = _new_stream_buffer(n, rate, d_in.device)
    _check_device_tensor(d_out, torch.uint8, "d_out")
    rc = lib().zc_compress(d_in.data_ptr(), n, int(rate), d_out.data_ptr(), d_out.numel(), _stream_handle(stream))
    if rc != ZC_OK:
        raise ZcError(rc, "zc_compress")
    return d_out


def zc_decompress(d_in, n, rate, d_out=None, stream=None):
    """uint8 CUDA tensor holding the compressed form of n values -> fp32 CUDA tensor."""
    _check_device_tensor(d_in, torch.uint8, "d_in")
    need = zc_compressed_size(n, rate)
    if need == 0 and n != 0:
        raise ZcError(ZC_ERR_RATE, "zc_decompress")
    if d_in.numel() < need:
        raise ValueError("d_in holds %d bytes, %d values at rate %d need %d" % (d_in.numel(), n, rate, need))
    if d_out is None:
        d_out = torch.empty(n, dtype=torch.float32, device=d_in.device)
    _check_device_tensor(d_out, torch.float32, "d_out")
    if d_out.numel() < n:
        raise ValueError("d_out holds %d values, need %d" % (d_out.numel(), n))
    rc = lib().zc_decompress(d_in.data_ptr(), int(n), int(rate), d_out.data_ptr(), _stream_handle(stream))
    if rc != ZC_OK:
        raise ZcError(rc, "zc_decompress")
    return d_out


def zc_reduce_compressed(d_in, n, rate, d_out=None, stream=None):
    """List of k uint8 CUDA tensors (compressed chunks of n values) -> compressed sum."""
    chunks = list(d_in)
    need = zc_compressed_size(n, rate)
    if need == 0 and n != 0:
        raise ZcError(ZC_ERR_RATE, "zc_reduce_compressed")
    for c in chunks:
        _check_device_tensor(c, torch.uint8, "every chunk")
        if c.numel() < need:
            raise ValueError("a chunk holds %d bytes, need %d" % (c.numel(), need))
    if d_out is None:
        device = chunks[0].device if chunks else torch.device("cuda")
        d_out = _new_stream_buffer(n, rate, device)
    _check_device_tensor(d_out, torch.uint8, "d_out")
    k = len(chunks)
    ptrs = (ctypes.c_void_p * max(k, 1))(*[c.data_ptr() for c in chunks])
    rc = lib().zc_reduce_compressed(ptrs, k, int(n), int(rate), d_out.data_ptr(), d_out.numel(),
                                    _stream_handle(stream))
    if rc != ZC_OK:
        raise ZcError(rc, "zc_reduce_compressed")
    return d_out


def _chunk_array(d_in, n, rate, what):
    chunks = list(d_in)
    need = zc_compressed_size(n, rate)
    if need == 0 and n != 0:
        raise ZcError(ZC_ERR_RATE, what)
    for c in chunks:
        _check_device_tensor(c, torch.uint8, "every chunk")
        if c.numel() < need:
            raise ValueError("a chunk holds %d bytes, need %d" % (c.numel(), need))
    return chunks, (ctypes.c_void_p * max(len(chunks), 1))(*[c.data_ptr() for c in chunks])


def _local_pointer(d_local, n):
    if d_local is None:
        return None
    _check_device_tensor(d_local, torch.float32, "d_local")
    if d_local.numel() < n:
        raise ValueError("d_local holds %d values, need %d" % (d_local.numel(), n))
    return d_local.data_ptr()


def zc_reduce_mixed(d_in, d_local, n, rate, d_out=None, stream=None):
    """k compressed chunks plus raw fp32 local values (or None) -> compressed sum."""
    chunks, ptrs = _chunk_array(d_in, n, rate, "zc_reduce_mixed")
    local = _local_pointer(d_local, n)
    if d_out is None:
        device = chunks[0].device if chunks else torch.device("cuda")
        d_out = _new_stream_buffer(n, rate, device)
    _check_device_tensor(d_out, torch.uint8, "d_out")
    rc = lib().zc_reduce_mixed(ptrs, len(chunks), local, int(n), int(rate), d_out.data_ptr(), d_out.numel(),
                               _stream_handle(stream))
    if rc != ZC_OK:
        raise ZcError(rc, "zc_reduce_mixed")
    return d_out


def zc_reduce_decompress(d_in, d_local, n, rate, d_out=None, stream=None):
    """k compressed chunks plus raw fp32 local values (or None) -> fp32 sum."""
    chunks, ptrs = _chunk_array(d_in, n, rate, "zc_reduce_decompress")
    local = _local_pointer(d_local, n)
    if d_out is None:
        device = chunks[0].device if chunks else torch.device("cuda")
        d_out = torch.empty(n, dtype=torch.float32, device=device)
    _check_device_tensor(d_out, torch.float32, "d_out")
    if d_out.numel() < n:
        raise ValueError("d_out holds %d values, need %d" % (d_out.numel(), n))
    rc = lib().zc_reduce_decompress(ptrs, len(chunks), local, int(n), int(rate), d_out.data_ptr(),
                                    _stream_handle(stream))
    if rc != ZC_OK:
        raise ZcError(rc, "zc_reduce_decompress")
    return d_out


def _half_dtype(t):
    if t.dtype == torch.bfloat16:
        return ZC_BF16
    if t.dtype == torch.float16:
        return ZC_F16
    raise TypeError("expected a bfloat16 or float16 tensor")


def zc_compress_half(d_in, rate, d_out=None, stream=None):
    """bfloat16 / float16 CUDA tensor -> uint8 CUDA tensor (same stream format as zc_compress)."""
    dtype = _half_dtype(d_in)
    _check_device_tensor(d_in, d_in.dtype, "d_in")
    n = d_in.numel()
    if d_out is None:
        d_out = _new_stream_buffer(n, rate, d_in.device)
    _check_device_tensor(d_out, torch.uint8, "d_out")
    rc = lib().zc_compress_half(d_in.data_ptr(), dtype, n, int(rate), d_out.data_ptr(), d_out.numel(),
                                _stream_handle(stream))
    if rc != ZC_OK:
        raise ZcError(rc, "zc_compress_half")
    return d_out


def zc_decompress_half(d_in, n, rate, dtype=None, d_out=None, stream=None):
    """Compressed stream -> bfloat16 / float16 CUDA tensor; give torch dtype or d_out."""
    _check_device_tensor(d_in, torch.uint8, "d_in")
    need = zc_compressed_size(n, rate)
    if need == 0 and n != 0:
        raise ZcError(ZC_ERR_RATE, "zc_decompress_half")
    if d_in.numel() < need:
        raise ValueError("d_in holds %d bytes, need %d" % (d_in.numel(), need))
    if d_out is None:
        d_out = torch.empty(n, dtype=dtype, device=d_in.device)
    code = _half_dtype(d_out)
    _check_device_tensor(d_out, d_out.dtype, "d_out")
    if d_out.numel() < n:
        raise ValueError("d_out holds %d values, need %d" % (d_out.numel(), n))
    rc = lib().zc_decompress_half(d_in.data_ptr(), int(n), int(rate), code, d_out.data_ptr(), _stream_handle(stream))
    if rc != ZC_OK:
        raise ZcError(rc, "zc_decompress_half")
    return d_out



def zc2d_rate_supported(rate):
    return bool(lib().zc2d_rate_supported(int(rate)))


def zc2d_compressed_size(rows, cols, rate):
    return int(lib().zc2d_compressed_size(int(rows), int(cols), int(rate)))


def zc2d_compress(d_in, rate, d_out=None, stream=None):
    """2-D fp32 CUDA tensor (rows x cols, row-major) -> uint8 CUDA tensor in format ZC-2D."""
    _check_device_tensor(d_in, torch.float32, "d_in")
    if d_in.dim() != 2:
        raise TypeError("d_in must be a matrix")
    rows, cols = d_in.shape
    if d_out is None:
        size = zc2d_compressed_size(rows, cols, rate)
        if size == 0 and rows * cols != 0:
            raise ZcError(ZC_ERR_RATE, "zc2d_compressed_size")
        d_out = torch.empty(size, dtype=torch.uint8, device=d_in.device)
    _check_device_tensor(d_out, torch.uint8, "d_out")
    rc = lib().zc2d_compress(d_in.data_ptr(), rows, cols, int(rate), d_out.data_ptr(), d_out.numel(),
                             _stream_handle(stream))
    if rc != ZC_OK:
        raise ZcError(rc, "zc2d_compress")
    return d_out


def zc2d_decompress(d_in, rows, cols, rate, d_out=None, stream=None):
    """uint8 CUDA tensor in format ZC-2D -> fp32 CUDA tensor of shape (rows, cols)."""
    _check_device_tensor(d_in, torch.uint8, "d_in")
    need = zc2d_compressed_size(rows, cols, rate)
    if need == 0 and rows * cols != 0:
        raise ZcError(ZC_ERR_RATE, "zc2d_decompress")
    if d_in.numel() < need:
        raise ValueError("d_in holds %d bytes, need %d" % (d_in.numel(), need))
    if d_out is None:
        d_out = torch.empty((rows, cols), dtype=torch.float32, device=d_in.device)
    _check_device_tensor(d_out, torch.float32, "d_out")
    if d_out.numel() < rows * cols:
        raise ValueError("d_out holds %d values, need %d" % (d_out.numel(), rows * cols))
    rc = lib().zc2d_decompress(d_in.data_ptr(), int(rows), int(cols), int(rate), d_out.data_ptr(),
                               _stream_handle(stream))
    if rc != ZC_OK:
        raise ZcError(rc, "zc2d_decompress")
    return d_out


def zc2d_compress_half(d_in, rate, d_out=None, stream=None):
    """2-D bfloat16 / float16 CUDA tensor -> uint8 CUDA tensor in format ZC-2D."""
    dtype = _half_dtype(d_in)
    _check_device_tensor(d_in, d_in.dtype, "d_in")
    if d_in.dim() != 2:
        raise TypeError("d_in must be a matrix")
    rows, cols = d_in.shape
    if d_out is None:
        size = zc2d_compressed_size(rows, cols, rate)
        if size == 0 and rows * cols != 0:
            raise ZcError(ZC_ERR_RATE, "zc2d_compressed_size")
        d_out = torch.empty(size, dtype=torch.uint8, device=d_in.device)
    _check_device_tensor(d_out, torch.uint8, "d_out")
    rc = lib().zc2d_compress_half(d_in.data_ptr(), dtype, rows, cols, int(rate), d_out.data_ptr(), d_out.numel(),
                                  _stream_handle(stream))
    if rc != ZC_OK:
        raise ZcError(rc, "zc2d_compress_half")
    return d_out


def zc2d_decompress_half(d_in, rows, cols, rate, dtype=None, d_out=None, stream=None):
    """Stream in format ZC-2D -> bfloat16 / float16 CUDA tensor of shape (rows, cols); give torch dtype or d_out."""
    _check_device_tensor(d_in, torch.uint8, "d_in")
    need = zc2d_compressed_size(rows, cols, rate)
    if need == 0 and rows * cols != 0:
        raise ZcError(ZC_ERR_RATE, "zc2d_decompress_half")
    if d_in.numel() < need:
        raise ValueError("d_in holds %d bytes, need %d" % (d_in.numel(), need))
    if d_out is None:
        d_out = torch.empty((rows, cols), dtype=dtype, device=d_in.device)
    code = _half_dtype(d_out)
    _check_device_tensor(d_out, d_out.dtype, "d_out")
    if d_out.numel() < rows * cols:
        raise ValueError("d_out holds %d values, need %d" % (d_out.numel(), rows * cols))
    rc = lib().zc2d_decompress_half(d_in.data_ptr(), int(rows), int(cols), int(rate), code, d_out.data_ptr(),
                                    _stream_handle(stream))
    if rc != ZC_OK:
        raise ZcError(rc, "zc2d_decompress_half")
    return d_out


def zc2d_reduce_compressed(d_in, rows, cols, rate, d_out=None, stream=None):
    """List of k uint8 CUDA tensors (compressed matrices of one shape) -> compressed sum."""
    chunks = list(d_in)
    need = zc2d_compressed_size(rows, cols, rate)
    if need == 0 and rows * cols != 0:
        raise ZcError(ZC_ERR_RATE, "zc2d_reduce_compressed")
    for c in chunks:
        _check_device_tensor(c, torch.uint8, "every chunk")
        if c.numel() < need:
            raise ValueError("a chunk holds %d bytes, need %d" % (c.numel(), need))
    if d_out is None:
        device = chunks[0].device if chunks else torch.device("cuda")
        d_out = torch.empty(need, dtype=torch.uint8, device=device)
    _check_device_tensor(d_out, torch.uint8, "d_out")
    ptrs = (ctypes.c_void_p * max(len(chunks), 1))(*[c.data_ptr() for c in chunks])
    rc = lib().zc2d_reduce_compressed(ptrs, len(chunks), int(rows), int(cols), int(rate), d_out.data_ptr(), d_out.numel(),
                                      _stream_handle(stream))
    if rc != ZC_OK:
        raise ZcError(rc, "zc2d_reduce_compressed")
    return d_out


def _chunks2d(d_in, rows, cols, rate, what):
    chunks = list(d_in)
    need = zc2d_compressed_size(rows, cols, rate)
    if need == 0 and rows * cols != 0:
        raise ZcError(ZC_ERR_RATE, what)
    for c in chunks:
        _check_device_tensor(c, torch.uint8, "every chunk")
        if c.numel() < need:
            raise ValueError("a chunk holds %d bytes, need %d" % (c.numel(), need))
    return chunks, need, (ctypes.c_void_p * max(len(chunks), 1))(*[c.data_ptr() for c in chunks])


def _local2d(d_local, rows, cols):
    if d_local is None:
        return None
    _check_device_tensor(d_local, torch.float32, "d_local")
    if tuple(d_local.shape) != (rows, cols):
        raise ValueError("d_local must have shape (%d, %d)" % (rows, cols))
    return d_local.data_ptr()


def zc2d_reduce_mixed(d_in, d_local, rows, cols, rate, d_out=None, stream=None):
    """k compressed matrices plus a raw fp32 matrix (or None) -> compressed sum."""
    chunks, need, ptrs = _chunks2d(d_in, rows, cols, rate, "zc2d_reduce_mixed")
    local = _local2d(d_local, rows, cols)
    if d_out is None:
        device = chunks[0].device if chunks else torch.device("cuda")
        d_out = torch.empty(need, dtype=torch.uint8, device=device)
    _check_device_tensor(d_out, torch.uint8, "d_out")
    rc = lib().zc2d_reduce_mixed(ptrs, len(chunks), local, int(rows), int(cols), int(rate), d_out.data_ptr(), d_out.numel(),
                                 _stream_handle(stream))
    if rc != ZC_OK:
        raise ZcError(rc, "zc2d_reduce_mixed")
    return d_out


def zc2d_reduce_decompress(d_in, d_local, rows, cols, rate, d_out=None, stream=None):
    """k compressed matrices plus a raw fp32 matrix (or None) -> fp32 sum of shape (rows, cols)."""
    chunks, need, ptrs = _chunks2d(d_in, rows, cols, rate, "zc2d_reduce_decompress")
    local = _local2d(d_local, rows, cols)
    if d_out is None:
        device = chunks[0].device if chunks else torch.device("cuda")
        d_out = torch.empty((rows, cols), dtype=torch.float32, device=device)
    _check_device_tensor(d_out, torch.float32, "d_out")
    if d_out.numel() < rows * cols:
        raise ValueError("d_out holds %d values, need %d" % (d_out.numel(), rows * cols))
    rc = lib().zc2d_reduce_decompress(ptrs, len(chunks), local, int(rows), int(cols), int(rate), d_out.data_ptr(),
                                      _stream_handle(stream))
    if rc != ZC_OK:
        raise ZcError(rc, "zc2d_reduce_decompress")
    return d_out


def zl_max_compressed_size(n):
    return int(lib().zl_max_compressed_size(int(n)))


def _check_words(t, what):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.element_size() == 4 and t.is_contiguous()):
        raise TypeError("%s must be a contiguous CUDA tensor of 32-bit items" % what)


def zl_compress(d_in, d_out=None, stream=None):
    """CUDA tensor of 32-bit items -> uint8 CUDA tensor of zl_max_compressed_size(n) bytes that
    starts with the lossless stream; zl_stream_bytes gives the stream's own length."""
    _check_words(d_in, "d_in")
    n = d_in.numel()
    if d_out is None:
        d_out = torch.empty(zl_max_compressed_size(n), dtype=torch.uint8, device=d_in.device)
    _check_device_tensor(d_out, torch.uint8, "d_out")
    rc = lib().zl_compress(d_in.data_ptr(), n, d_out.data_ptr(), d_out.numel(), _stream_handle(stream))
    if rc != ZC_OK:
        raise ZcError(rc, "zl_compress")
    return d_out


def zl_stream_bytes(d_stream, stream=None):
    """Length of the lossless stream at the start of d_stream (waits for the stream's work)."""
    _check_device_tensor(d_stream, torch.uint8, "d_stream")
    if d_stream.numel() < 32:
        raise ValueError("d_stream is shorter than a header")
    size = ctypes.c_size_t(0)
    rc = lib().zl_stream_bytes(d_stream.data_ptr(), ctypes.byref(size), _stream_handle(stream))
    if rc != ZC_OK:
        raise ZcError(rc, "zl_stream_bytes")
    return int(size.value)


def zl_decompress(d_in, n, d_out=None, dtype=torch.float32, stream=None):
    """Lossless stream (uint8 CUDA tensor, at least the stream's length) -> n 32-bit items."""
    _check_device_tensor(d_in, torch.uint8, "d_in")
    if d_out is None:
        d_out = torch.empty(int(n), dtype=dtype, device=d_in.device)
    _check_words(d_out, "d_out")
    if d_out.numel() < n:
        raise ValueError("d_out holds %d items, need %d" % (d_out.numel(), n))
    rc = lib().zl_decompress(d_in.data_ptr(), d_in.numel(), int(n), d_out.data_ptr(), _stream_handle(stream))
    if rc != ZC_OK:
        raise ZcError(rc, "zl_decompress")
    return d_out


def _check_halves(t, what):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.element_size() == 2 and t.is_contiguous()):
        raise TypeError("%s must be a contiguous CUDA tensor of 16-bit items" % what)


def zl_compress16(d_in, d_out=None, stream=None):
    """CUDA tensor of 16-bit items (bfloat16, float16, int16) -> uint8 CUDA tensor that starts with the
    lossless stream of the items taken as the upper halves of 32-bit words."""
    _check_halves(d_in, "d_in")
    n = d_in.numel()
    if d_out is None:
        d_out = torch.empty(zl_max_compressed_size(n), dtype=torch.uint8, device=d_in.device)
    _check_device_tensor(d_out, torch.uint8, "d_out")
    rc = lib().zl_compress16(d_in.data_ptr(), n, d_out.data_ptr(), d_out.numel(), _stream_handle(stream))
    if rc != ZC_OK:
        raise ZcError(rc, "zl_compress16")
    return d_out


def zl_decompress16(d_in, n, d_out=None, dtype=torch.bfloat16, stream=None):
    """Lossless stream -> the upper halves of its n words as 16-bit items."""
    _check_device_tensor(d_in, torch.uint8, "d_in")
    if d_out is None:
        d_out = torch.empty(int(n), dtype=dtype, device=d_in.device)
    _check_halves(d_out, "d_out")
    if d_out.numel() < n:
        raise ValueError("d_out holds %d items, need %d" % (d_out.numel(), n))
    rc = lib().zl_decompress16(d_in.data_ptr(), d_in.numel(), int(n), d_out.data_ptr(), _stream_handle(stream))
    if rc != ZC_OK:
        raise ZcError(rc, "zl_decompress16")
    return d_out
