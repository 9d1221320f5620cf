/*
 * zc.h -- C ABI of libzc: fixed-rate compression of collective message buffers
 * on MI355X (gfx950).
 *
 * The paper accelerates 3D-parallel + ZeRO LLM training by running every
 * collective on compressed messages: a lossy fixed-rate codec of the ZFP family,
 * at a low rate for data-parallel gradients and a higher rate for
 * tensor/pipeline/ZeRO traffic (Sec. II-A, Sec. III-B and Table III, rates 8, 16,
 * 24 in Sec. IV-C and IV-F), with the all-reduce built from a compressed
 * reduce-scatter and all-gather (Sec. IV-A).  This library is the per-GPU part of
 * that: compress a message, decompress a message, and the
 * decompress-accumulate-recompress step of the reduce-scatter.
 *
 * Codec ("ZC-1"): the buffer is cut into blocks of 4 consecutive fp32 values; each
 * block becomes exactly 4*rate bits = rate/2 bytes, stored back to back (block j at
 * byte j*rate/2): one header byte (biased shared exponent, 0 = all-zero block) and
 * 4*rate-8 payload bits produced by block-floating-point conversion, a reversible
 * integer lifting transform, negabinary mapping and embedded bit-plane coding.
 * A buffer whose length is not a multiple of 4 is padded by repeating its last
 * value; the pad is dropped on decompression.
 *
 * Conventions for every call below
 *   - Pointers named d_* are DEVICE pointers, owned by the caller, 16-byte aligned.
 *     The library neither allocates, frees nor keeps them.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     enqueue kernels on it and return without synchronising; buffers must stay
 *     valid until that work has finished.
 *   - Return value: ZC_OK or a negative error code; on error nothing is launched.
 *   - n is a count of fp32 values.  n == 0 is valid and does nothing.
 *   - Values that are not finite are outside the contract (the result is
 *     unspecified, but no access leaves the buffers).
 *   - The library allocates nothing, keeps no state between calls and reads no
 *     environment variable; calls on different streams may run concurrently.
 */
#ifndef ZC_H
#define ZC_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  ZC_OK = 0,
  ZC_ERR_NULL = -1,     /* a required pointer is NULL */
  ZC_ERR_RATE = -2,     /* rate not in {4,8,...,32} (zc2d_*: not in {2,4,8,16}) */
  ZC_ERR_SIZE = -3,     /* n too large for this build (more than 2^40 values) */
  ZC_ERR_CAPACITY = -4, /* out_cap smaller than zc_compressed_size(n, rate) */
  ZC_ERR_K = -5,        /* k outside [1, 16] */
  ZC_ERR_ALIGN = -6,    /* a device pointer is not 16-byte aligned */
  ZC_ERR_LAUNCH = -7,   /* the HIP runtime refused the launch */
  ZC_ERR_DTYPE = -8,    /* dtype is not ZC_BF16 or ZC_F16 */
  ZC_ERR_STREAM = -9    /* zl_stream_bytes: the buffer does not start with a complete lossless stream */
};

/* Element types of a message buffer.  The fp32 calls take no dtype argument. */
enum zc_dtype { ZC_F32 = 0, ZC_BF16 = 1, ZC_F16 = 2 };

/* Message classes of Table I / Table III. */
enum zc_class {
  ZC_DP_GRADIENT = 0,   /* data-parallel all-reduce */
  ZC_TP_ACTIVATION = 1, /* tensor-parallel all-reduce / all-gather */
  ZC_PP_ACTIVATION = 2, /* pipeline point-to-point */
  ZC_ZERO_PARAM = 3,    /* ZeRO-1 parameter all-gather */
  ZC_OPT_STATE = 4      /* ZeRO-1 reduce-scatter / optimizer-state traffic */
};

/* The two hybrid schemes: fixed-rate codec everywhere at two rates (Sec. III-B, Table
 * III), or lossless codec for model-parallel and ZeRO traffic and the fixed-rate codec for
 * data-parallel gradients (Sec. III-A, Table II). */
enum zc_scheme { ZC_SCHEME_ZHYBRID = 0, ZC_SCHEME_MZHYBRID = 1 };
enum zc_codec { ZC_CODEC_FIXED_RATE = 0, ZC_CODEC_LOSSLESS = 1 };

/* Library version, major*100 + minor. */
int zc_version(void);

/* Static description of an error code (never NULL). */
const char* zc_strerror(int code);

/* 1 if `rate` (bits per value) is supported: multiples of 4 from 4 to 32. */
int zc_rate_supported(int rate);

/* Rate of the hybrid scheme of Sec. III-B (Table III): low rate for
 * data-parallel gradients (8, as in Sec. IV-F), high rate (16) for everything
 * else.  Returns 0 for an unknown class. */
int zc_rate_for_class(enum zc_class c);

/* Codec for a message class under a scheme: ZC_CODEC_FIXED_RATE (the zc_* and zc2d_*
 * calls) with its rate in *rate, or ZC_CODEC_LOSSLESS (the zl_* calls) with *rate = 0.
 * ZHybrid: the rates of zc_rate_for_class.  MZHybrid: lossless for every class except
 * data-parallel gradients, which keep the low rate (8; Sec. IV-E also ran 16).  Returns -1
 * for an unknown scheme or class.  `rate` is a host pointer and may be NULL. */
int zc_codec_for_class(enum zc_scheme s, enum zc_class c, int* rate);

/* Bytes of the compressed form of n values: ceil(n/4) * rate/2, which is
 * n*rate/8 when 4 divides n.  0 if the rate is unsupported. */
size_t zc_compressed_size(size_t n, int rate);

/* Compress d_in[0..n) into d_out[0..zc_compressed_size(n,rate)).
 * d_out must not overlap d_in. */
int zc_compress(const float* d_in, size_t n, int rate, void* d_out, size_t out_cap, void* stream);

/* Decompress into d_out[0..n).  d_in holds zc_compressed_size(n,rate) bytes and may
 * contain arbitrary bytes (every byte string decodes to something).  d_out must not
 * overlap d_in. */
int zc_decompress(const void* d_in, size_t n, int rate, float* d_out, void* stream);

/* The reduce-scatter step (Sec. IV-A): d_in is a HOST array of k device pointers to
 * compressed chunks of n values each (same rate).  Writes to d_out the compressed
 * form of the element-wise fp32 sum ((x_0 + x_1) + x_2) + ... of the decompressed
 * chunks; nothing but the k inputs and the output touches device memory.  The
 * pointer array is read before the call returns.  d_out may be the same buffer as
 * one of the inputs (each block is read before it is written) but must not
 * partially overlap any.  The chunks may hold arbitrary bytes: the result is that of
 * decompressing each and adding, also where a decoded value is infinite (a sum that
 * is not a number makes that block's output unspecified).  Re-encoding at every hop
 * of a ring needs rate 8 or more to stay accurate: at rate 4 the error of the running
 * sum about doubles per hop, while one k-way call re-encodes once. */
int zc_reduce_compressed(const void* const* d_in, int k, size_t n, int rate, void* d_out,
                         size_t out_cap, void* stream);

/* A ring hop of the compressed reduce-scatter in which this rank's own contribution
 * is still raw fp32 (Sec. IV-A: every rank adds its gradients to the chunk it received
 * and forwards the result): writes the compressed form of
 * ((x_0 + ... + x_{k-1}) + local), x_j = decompressed chunk j, every add in fp32.
 * d_in as in zc_reduce_compressed (k in [1, 16]); d_local holds n fp32 values and may
 * be NULL, which makes this call zc_reduce_compressed.  d_out may be one of the inputs
 * d_in[j] but must not overlap d_local. */
int zc_reduce_mixed(const void* const* d_in, int k, const float* d_local, size_t n, int rate,
                    void* d_out, size_t out_cap, void* stream);

/* The last hop, where the sum is consumed uncompressed: d_out[i] =
 * ((x_0 + ... + x_{k-1}) + local)[i] as fp32, nothing re-encoded.  d_local may be NULL;
 * with k = 1 and d_local = NULL this is zc_decompress.  d_out (n values) may be the same
 * buffer as d_local (each value is read before it is written) but must not overlap
 * any d_in[j]. */
int zc_reduce_decompress(const void* const* d_in, int k, const float* d_local, size_t n, int rate,
                         float* d_out, void* stream);

/* Half-precision messages (the paper does not state its message precision; LLM
 * training traffic is usually bf16 or fp16).  d_in holds n values of `dtype` (ZC_BF16
 * or ZC_F16, 2 bytes each).  Every value is widened to fp32, which is exact, and then
 * compressed exactly as zc_compress would: the stream is the same format and can be fed
 * to every other call. */
int zc_compress_half(const void* d_in, int dtype, size_t n, int rate, void* d_out, size_t out_cap,
                     void* stream);

/* Decompress to n values of `dtype`: what zc_decompress would produce, each value
 * rounded to the nearest bf16 / fp16 (ties to even; magnitudes beyond the largest
 * finite value become infinity). */
int zc_decompress_half(const void* d_in, size_t n, int rate, int dtype, void* d_out, void* stream);

/*
 * Matrix-shaped messages, format "ZC-2D": the same codec family (Sec. II-A, Sec.
 * III-B) on blocks of 4 x 4 values, for weight-matrix gradients and [tokens x hidden]
 * activations, whose structure runs in both directions (the low-rank remark of Sec. I).
 * A row-major rows x cols fp32 matrix is cut into blocks (bi, bj) = rows 4bi..4bi+3,
 * columns 4bj..4bj+3, stored in row-major block order, each exactly 16*rate bits =
 * 2*rate bytes: one header byte (biased shared exponent of the 16 values, 0 = all-zero
 * block) and 16*rate-8 payload bits from block-floating-point conversion with 27
 * fraction bits, the lifting transform of ZC-1 along rows and then along columns,
 * coefficients ordered by total frequency, negabinary mapping and embedded bit-plane
 * coding over 16 coefficients.  Blocks that stick out of the matrix are filled by
 * repeating the last row / column; the fill is dropped on decompression.  The
 * conventions at the top of this file apply (device pointers, 16-byte aligned, stream,
 * error codes); ZC_ERR_RATE here means a rate outside {2, 4, 8, 16}, ZC_ERR_SIZE a
 * matrix of more than 2^40 values.  rows == 0 or cols == 0 is valid and does nothing.
 */

/* 1 if `rate` (bits per value) is supported by the zc2d_* calls: 2, 4, 8, 16. */
int zc2d_rate_supported(int rate);

/* Bytes of the compressed form of a rows x cols matrix:
 * ceil(rows/4) * ceil(cols/4) * 2*rate.  0 if the rate is unsupported. */
size_t zc2d_compressed_size(size_t rows, size_t cols, int rate);

/* Compress the row-major matrix d_in[rows*cols] into
 * d_out[0..zc2d_compressed_size(rows,cols,rate)).  d_out must not overlap d_in. */
int zc2d_compress(const float* d_in, size_t rows, size_t cols, int rate, void* d_out, size_t out_cap,
                  void* stream);

/* Decompress into the row-major matrix d_out[rows*cols].  d_in holds
 * zc2d_compressed_size(rows,cols,rate) bytes and may contain arbitrary bytes.  d_out
 * must not overlap d_in. */
int zc2d_decompress(const void* d_in, size_t rows, size_t cols, int rate, float* d_out, void* stream);

/* Half-precision matrices (bf16 / fp16, 2 bytes per value; the usual precision of
 * [tokens x hidden] activations): every value is widened to fp32, which is exact, and the
 * matrix is compressed exactly as zc2d_compress would; the stream is an ordinary ZC-2D
 * stream.  dtype is ZC_BF16 or ZC_F16 (else ZC_ERR_DTYPE). */
int zc2d_compress_half(const void* d_in, int dtype, size_t rows, size_t cols, int rate, void* d_out, size_t out_cap,
                       void* stream);

/* Decompress to a half-precision matrix: what zc2d_decompress would produce, each value
 * rounded to the nearest bf16 / fp16 (ties to even; magnitudes beyond the largest finite
 * value become infinity). */
int zc2d_decompress_half(const void* d_in, size_t rows, size_t cols, int rate, int dtype, void* d_out, void* stream);

/* The reduce-scatter step (Sec. IV-A) on matrix-shaped messages: d_in is a HOST array of
 * k device pointers (k in [1, 16]) to compressed matrices of the same shape and rate.
 * Writes to d_out the compressed form of the element-wise fp32 sum ((x_0 + x_1) + x_2) +
 * ... of the decompressed matrices; only the k inputs and the output touch device memory.
 * The pointer array is read before the call returns.  d_out may be the same buffer as one
 * of the inputs (each block is read before it is written) but must not partially overlap
 * any. */
int zc2d_reduce_compressed(const void* const* d_in, int k, size_t rows, size_t cols, int rate, void* d_out,
                           size_t out_cap, void* stream);

/* The ring hops of the reduce-scatter on matrix-shaped messages, as zc_reduce_mixed and
 * zc_reduce_decompress (Sec. IV-A): the compressed form, respectively the fp32 matrix, of
 * ((x_0 + ... + x_{k-1}) + local), x_j the decompressed matrix j, local a raw row-major fp32
 * matrix of the same shape that may be NULL.  The compressed output may be one of the inputs
 * d_in[j]; the fp32 output may be the same buffer as d_local; no other overlap. */
int zc2d_reduce_mixed(const void* const* d_in, int k, const float* d_local, size_t rows, size_t cols, int rate, void* d_out,
                      size_t out_cap, void* stream);
int zc2d_reduce_decompress(const void* const* d_in, int k, const float* d_local, size_t rows, size_t cols, int rate,
                           float* d_out, void* stream);

/*
 * Lossless messages, format "ZL-1": the role the paper's first hybrid scheme gives to a
 * lossless codec of the MPC kind on model-parallel traffic (Sec. II-A, Sec. III-A and its
 * table of collectives).  The message is n 32-bit words (fp32 values as bit patterns; any
 * pattern, NaN and infinities included, comes back unchanged).  Chunks of 8192 words are
 * coded on their own: a chunk is 256 groups of 32 words (word j of group g is chunk word
 * 1024*(j/4) + 4*g + j%4); each word of a group becomes sign | (largest magnitude of the
 * group - its magnitude), the 32 residuals are bit-transposed and the zero planes dropped.
 * Stream: header (32 bytes: u32 magic "ZL01", u32 chunks, u64 n, u64 total bytes, u64 zero),
 * a table of one u64 per chunk (binary 10 in the top two bits, below them the byte offset
 * in the payload at which the chunk ends), then per chunk 256 references, 256 plane bitmaps
 * and the non-zero planes.  The size of a stream depends on the data; it is at most
 * zl_max_compressed_size(n) and is recorded in the header.  Device pointers, 16-byte
 * aligned; the conventions at the top of this file apply.
 */

/* Capacity d_out must have for a message of n words: the size of the stream when no plane
 * is dropped, 32 + ceil(n/8192) * (8 + 2048 + 32768).  0 if n exceeds 2^40. */
size_t zl_max_compressed_size(size_t n);

/* Compress d_in[0..n) (32-bit words) into a stream at d_out.  Bytes of d_out beyond the
 * stream's own length are left as they were.  d_out must not overlap d_in.  Uses no memory
 * besides d_in and d_out, and may be captured in a HIP graph. */
int zl_compress(const void* d_in, size_t n, void* d_out, size_t out_cap, void* stream);

/* Length in bytes of the stream at d_stream, read from its header into *h_bytes (a HOST
 * pointer).  Waits for the work queued on `stream` before it returns.  ZC_ERR_STREAM if the
 * buffer does not start with a complete stream. */
int zl_stream_bytes(const void* d_stream, size_t* h_bytes, void* stream);

/* Decompress the stream in d_in[0..in_bytes) into d_out[0..n).  n must be the message
 * length the stream was made from, and in_bytes at least the stream's length; for anything
 * else the output is unspecified, but no access leaves d_in[0..in_bytes) or d_out[0..n).
 * ZC_ERR_CAPACITY if in_bytes cannot even hold the header and table for n words. */
int zl_decompress(const void* d_in, size_t in_bytes, size_t n, void* d_out, void* stream);

/* 16-bit messages (bf16, fp16 or anything else of that width; the paper does not state what
 * its messages hold): d_in holds n 16-bit words, which are coded as the n 32-bit words
 * v << 16, so the stream is an ordinary ZL-1 stream of n words (for bf16: of the values
 * widened to fp32) and every pattern comes back.  The empty lower halves cost nothing in the
 * stream.  Otherwise as zl_compress. */
int zl_compress16(const void* d_in, size_t n, void* d_out, size_t out_cap, void* stream);

/* As zl_decompress, but writes the upper halves of the n decoded words to d_out (n 16-bit
 * words); for a stream made by zl_compress16 the lower halves are zero. */
int zl_decompress16(const void* d_in, size_t in_bytes, size_t n, void* d_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ZC_H */
