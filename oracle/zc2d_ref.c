/*
 * zc2d_ref.c -- reference CPU codec for format "ZC-2D".  TEST INFRASTRUCTURE ONLY.
 *
 * The same codec family as zc_ref.c (the paper's lossy fixed-rate ZFP-kind
 * compressor, Sec. II-A, Sec. III-B), applied to matrix-shaped messages in
 * blocks of 4 x 4 values: gradients of weight matrices and [tokens x hidden]
 * activations have structure in both directions (the paper's low-rank remark
 * in Sec. I), which 1-D blocks cannot see, and one header per 16 values
 * instead of per 4 leaves more of a low rate for data.  The paper gives no
 * internals; everything below is a stated reading, listed in the design
 * notes.  Nothing here is shared with the HIP kernels.
 *
 * Format.  A row-major matrix rows x cols of fp32 is cut into blocks of 4 x 4
 * (block (bi,bj) = rows 4bi..4bi+3, columns 4bj..4bj+3), stored in row-major
 * block order, each exactly 16*rate bits = 2*rate bytes: one header byte
 * (biased shared exponent, 0 = all-zero block) and 16*rate-8 payload bits,
 * stream bit t in bit (t mod 8) of byte t/8.  Blocks that stick out of the
 * matrix are filled by repeating the last valid row / column; the decoder
 * drops the fill.
 *   1. shared exponent e of the 16 values, as in the 1-D format (clamped at
 *      -126), header E = e + 127;
 *   2. q = trunc(x * 2^(27 - e)): one fraction bit fewer than in 1-D, because
 *      the transform is applied twice;
 *   3. the reversible 1-D lifting transform (zc_ref_fwd_lift) on each of the 4
 *      rows, then on each of the 4 columns;
 *   4. coefficients ordered by total sequency (row frequency i + column
 *      frequency j, ties by smaller i), negabinary words;
 *   5. the embedded bit-plane code of the 1-D format with 16 coefficients in
 *      place of 4: per plane the bits of the n coefficients already
 *      significant, then group tests (group bit; if 1, unary search for the
 *      first one, implied at the last index), cut at the budget.
 * The decoder mirrors this; a group known to hold a one that the budget cut
 * before it was located gets the one at the lowest index still possible.
 *
 * Parity status: pinned by tests/test_oracle_2d.py.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#define ZC2D_FRACTION_BITS 27
#define ZC2D_COEFFS 16

/* pinned 1-D building blocks from zc_ref.c */
float zc_ref_widen(uint16_t h, int dtype);
uint16_t zc_ref_narrow(float f, int dtype);
void zc_ref_fwd_lift(int32_t v[4]);
void zc_ref_inv_lift(int32_t v[4]);
uint32_t zc_ref_negabinary(int32_t c);
int32_t zc_ref_inv_negabinary(uint32_t u);

enum { ZC2D_OK = 0, ZC2D_ERR_NULL = -1, ZC2D_ERR_RATE = -2, ZC2D_ERR_CAPACITY = -4, ZC2D_ERR_K = -5 };

int zc2d_ref_rate_supported(int rate) { return rate >= 1 && rate <= 32; }

size_t zc2d_ref_compressed_size(size_t rows, size_t cols, int rate) {
  if (!zc2d_ref_rate_supported(rate)) return 0;
  return ((rows + 3) / 4) * ((cols + 3) / 4) * (size_t)(2 * rate);
}

/* ---- coefficient order -------------------------------------------------- */

/* order[c] = 4*i + j of the c-th coefficient (i = row frequency after the
 * column pass, j = column frequency after the row pass): ascending i + j,
 * ties by ascending i. */
void zc2d_ref_order(int order[16]) {
  int c = 0;
  for (int s = 0; s <= 6; ++s)
    for (int i = 0; i < 4; ++i) {
      int j = s - i;
      if (j >= 0 && j < 4) order[c++] = 4 * i + j;
    }
}

/* ---- stages ---------------------------------------------------------------- */

int zc2d_ref_block_exponent(const float x[16]) {
  int any = 0, emax = 0;
  for (int i = 0; i < 16; ++i)
    if (x[i] != 0.0f) {
      int eps;
      (void)frexpf(x[i], &eps);
      if (!any || eps > emax) emax = eps;
      any = 1;
    }
  if (!any) return 0;
  if (emax < -126) emax = -126;
  return emax + 127;
}

/* q_i = x_i * 2^(27 - e), truncated toward zero.  The product is exact in double. */
void zc2d_ref_quantise(const float x[16], int E, int32_t q[16]) {
  for (int i = 0; i < 16; ++i)
    q[i] = (int32_t)trunc(ldexp((double)x[i], ZC2D_FRACTION_BITS - (E - 127)));
}

/* x_i = float(q_i) * 2^(e - 27): int -> fp32 with round-to-nearest-even, then an IEEE
 * scaling by a power of two (rounds a second time only for subnormal results). */
void zc2d_ref_dequantise(const int32_t q[16], int E, float x[16]) {
  for (int i = 0; i < 16; ++i) x[i] = ldexpf((float)q[i], (E - 127) - ZC2D_FRACTION_BITS);
}

/* v is the 4x4 block, row-major: lifting along each row, then along each column. */
void zc2d_ref_fwd_transform(int32_t v[16]) {
  for (int r = 0; r < 4; ++r) zc_ref_fwd_lift(v + 4 * r);
  for (int c = 0; c < 4; ++c) {
    int32_t t[4] = {v[c], v[4 + c], v[8 + c], v[12 + c]};
    zc_ref_fwd_lift(t);
    v[c] = t[0]; v[4 + c] = t[1]; v[8 + c] = t[2]; v[12 + c] = t[3];
  }
}

void zc2d_ref_inv_transform(int32_t v[16]) {
  for (int c = 0; c < 4; ++c) {
    int32_t t[4] = {v[c], v[4 + c], v[8 + c], v[12 + c]};
    zc_ref_inv_lift(t);
    v[c] = t[0]; v[4 + c] = t[1]; v[8 + c] = t[2]; v[12 + c] = t[3];
  }
  for (int r = 0; r < 4; ++r) zc_ref_inv_lift(v + 4 * r);
}

/* Embedded coder over 16 words.  bits[] gets one stream bit per element. */
int zc2d_ref_encode_planes(const uint32_t u[16], int budget, uint8_t *bits) {
  int left = budget, w = 0, n = 0;
  for (int t = 0; t < budget; ++t) bits[t] = 0;
  for (int k = 31; k >= 0 && left > 0; --k) {
    int p[16];
    for (int i = 0; i < 16; ++i) p[i] = (u[i] >> k) & 1;
    for (int i = 0; i < n && left > 0; ++i) { bits[w++] = (uint8_t)p[i]; --left; }
    int i = n;
    while (i < 16 && left > 0) {
      int g = 0;
      for (int j = i; j < 16; ++j) g |= p[j];
      bits[w++] = (uint8_t)g; --left;
      if (!g) break;
      while (i < 15 && left > 0) {
        bits[w++] = (uint8_t)p[i]; --left;
        if (p[i]) break;
        ++i;
      }
      ++i;
    }
    n = i;
  }
  return w;
}

void zc2d_ref_decode_planes(const uint8_t *bits, int budget, uint32_t u[16]) {
  int left = budget, r = 0, n = 0;
  for (int i = 0; i < 16; ++i) u[i] = 0;
  for (int k = 31; k >= 0 && left > 0; --k) {
    for (int i = 0; i < n && left > 0; ++i) {
      if (bits[r++]) u[i] |= 1u << k;
      --left;
    }
    int i = n;
    while (i < 16 && left > 0) {
      int g = bits[r++]; --left;
      if (!g) break;
      while (i < 15 && left > 0) {
        int b = bits[r++]; --left;
        if (b) break;
        ++i;
      }
      u[i] |= 1u << k;
      ++i;
    }
    n = i;
  }
}

/* ---- one block ---------------------------------------------------------- */

static void put_bit(uint8_t *s, size_t t, int bit) {
  if (bit) s[t >> 3] = (uint8_t)(s[t >> 3] | (1u << (t & 7)));
  else s[t >> 3] = (uint8_t)(s[t >> 3] & ~(1u << (t & 7)));
}
static int get_bit(const uint8_t *s, size_t t) { return (s[t >> 3] >> (t & 7)) & 1; }

void zc2d_ref_encode_block(const float x[16], int rate, uint8_t *out /* 2*rate bytes */) {
  const int B = 16 * rate, budget = B - 8;
  memset(out, 0, (size_t)(2 * rate));
  int E = zc2d_ref_block_exponent(x);
  if (E == 0) return;
  out[0] = (uint8_t)E;
  int32_t q[16];
  zc2d_ref_quantise(x, E, q);
  zc2d_ref_fwd_transform(q);
  int order[16];
  zc2d_ref_order(order);
  uint32_t u[16];
  for (int c = 0; c < 16; ++c) u[c] = zc_ref_negabinary(q[order[c]]);
  uint8_t bits[16 * 32];
  zc2d_ref_encode_planes(u, budget, bits);
  for (int t = 0; t < budget; ++t) put_bit(out, (size_t)(8 + t), bits[t]);
}

void zc2d_ref_decode_block(const uint8_t *in, int rate, float x[16]) {
  const int budget = 16 * rate - 8;
  int E = in[0];
  if (E == 0) { for (int i = 0; i < 16; ++i) x[i] = 0.0f; return; }
  uint8_t bits[16 * 32];
  for (int t = 0; t < budget; ++t) bits[t] = (uint8_t)get_bit(in, (size_t)(8 + t));
  uint32_t u[16];
  zc2d_ref_decode_planes(bits, budget, u);
  int order[16];
  zc2d_ref_order(order);
  int32_t q[16];
  for (int c = 0; c < 16; ++c) q[order[c]] = zc_ref_inv_negabinary(u[c]);
  zc2d_ref_inv_transform(q);
  zc2d_ref_dequantise(q, E, x);
}

/* ---- whole matrices (host pointers) -------------------------------------- */

int zc2d_ref_compress(const float *in, size_t rows, size_t cols, int rate, void *out, size_t out_cap) {
  if (!zc2d_ref_rate_supported(rate)) return ZC2D_ERR_RATE;
  if (rows == 0 || cols == 0) return ZC2D_OK;
  if (!in || !out) return ZC2D_ERR_NULL;
  if (out_cap < zc2d_ref_compressed_size(rows, cols, rate)) return ZC2D_ERR_CAPACITY;
  size_t bc = (cols + 3) / 4, br = (rows + 3) / 4;
  for (size_t bi = 0; bi < br; ++bi)
    for (size_t bj = 0; bj < bc; ++bj) {
      float x[16];
      for (int r = 0; r < 4; ++r)
        for (int c = 0; c < 4; ++c) {
          size_t rr = 4 * bi + (size_t)r, cc = 4 * bj + (size_t)c;
          if (rr >= rows) rr = rows - 1;   /* repeat the last valid row / column */
          if (cc >= cols) cc = cols - 1;
          x[4 * r + c] = in[rr * cols + cc];
        }
      zc2d_ref_encode_block(x, rate, (uint8_t *)out + (bi * bc + bj) * (size_t)(2 * rate));
    }
  return ZC2D_OK;
}

int zc2d_ref_decompress(const void *in, size_t rows, size_t cols, int rate, float *out) {
  if (!zc2d_ref_rate_supported(rate)) return ZC2D_ERR_RATE;
  if (rows == 0 || cols == 0) return ZC2D_OK;
  if (!in || !out) return ZC2D_ERR_NULL;
  size_t bc = (cols + 3) / 4, br = (rows + 3) / 4;
  for (size_t bi = 0; bi < br; ++bi)
    for (size_t bj = 0; bj < bc; ++bj) {
      float x[16];
      zc2d_ref_decode_block((const uint8_t *)in + (bi * bc + bj) * (size_t)(2 * rate), rate, x);
      for (int r = 0; r < 4; ++r)
        for (int c = 0; c < 4; ++c) {
          size_t rr = 4 * bi + (size_t)r, cc = 4 * bj + (size_t)c;
          if (rr < rows && cc < cols) out[rr * cols + cc] = x[4 * r + c];
        }
    }
  return ZC2D_OK;
}

/* The reduce-scatter step of the compressed all-reduce (Sec. IV-A) on matrix-shaped
 * messages: decode the k incoming matrices block by block, add them element by element
 * in fp32 in index order ((d0 + d1) + d2) + ..., and encode the sum.  The result is
 * compress(sum): where a block sticks out of the matrix it is filled with the last valid
 * row / column of the sum, not with the sum of the inputs' fills.  `out` may be the
 * same buffer as in[0]. */
int zc2d_ref_reduce_compressed(const void *const *in, int k, size_t rows, size_t cols, int rate,
                               void *out, size_t out_cap) {
  if (!zc2d_ref_rate_supported(rate)) return ZC2D_ERR_RATE;
  if (k < 1 || k > 16) return ZC2D_ERR_K;
  if (rows == 0 || cols == 0) return ZC2D_OK;
  if (!in || !out) return ZC2D_ERR_NULL;
  for (int c = 0; c < k; ++c)
    if (!in[c]) return ZC2D_ERR_NULL;
  if (out_cap < zc2d_ref_compressed_size(rows, cols, rate)) return ZC2D_ERR_CAPACITY;
  size_t bc = (cols + 3) / 4, br = (rows + 3) / 4;
  for (size_t bi = 0; bi < br; ++bi)
    for (size_t bj = 0; bj < bc; ++bj) {
      size_t at = (bi * bc + bj) * (size_t)(2 * rate);
      float s[16], d[16];
      zc2d_ref_decode_block((const uint8_t *)in[0] + at, rate, s);
      for (int c = 1; c < k; ++c) {
        zc2d_ref_decode_block((const uint8_t *)in[c] + at, rate, d);
        for (int i = 0; i < 16; ++i) {
          volatile float t = s[i] + d[i]; /* one fp32 rounding per add */
          s[i] = t;
        }
      }
      size_t rv = rows - 4 * bi < 4 ? rows - 4 * bi : 4, cv = cols - 4 * bj < 4 ? cols - 4 * bj : 4;
      float f[16];
      for (size_t r = 0; r < 4; ++r)
        for (size_t q = 0; q < 4; ++q) f[4 * r + q] = s[4 * (r < rv ? r : rv - 1) + (q < cv ? q : cv - 1)];
      zc2d_ref_encode_block(f, rate, (uint8_t *)out + at);
    }
  return ZC2D_OK;
}

/* Sum of block (bi, bj) over the k inputs and, if `local` is given, the raw local values
 * added last: ((d0 + d1) + ... + d_{k-1}) + x, one fp32 rounding per add.  Positions outside
 * the matrix take no local value; they are filled or dropped by the caller. */
static void sum_block2d(const void *const *in, int k, const float *local, size_t rows, size_t cols,
                        size_t bi, size_t bj, int rate, float s[16]) {
  size_t bc = (cols + 3) / 4, at = (bi * bc + bj) * (size_t)(2 * rate);
  float d[16];
  zc2d_ref_decode_block((const uint8_t *)in[0] + at, rate, s);
  for (int c = 1; c < k; ++c) {
    zc2d_ref_decode_block((const uint8_t *)in[c] + at, rate, d);
    for (int i = 0; i < 16; ++i) {
      volatile float t = s[i] + d[i];
      s[i] = t;
    }
  }
  if (local)
    for (size_t r = 0; r < 4; ++r)
      for (size_t q = 0; q < 4; ++q) {
        size_t rr = 4 * bi + r, cc = 4 * bj + q;
        if (rr < rows && cc < cols) {
          volatile float t = s[4 * r + q] + local[rr * cols + cc];
          s[4 * r + q] = t;
        }
      }
}

/* A ring hop whose local contribution is still a raw fp32 matrix (Sec. IV-A: each rank adds
 * its own gradients to what it received before forwarding): out = compress(((d0 + ... +
 * d_{k-1}) + local)), the edge fill taken from that sum.  local may be NULL. */
int zc2d_ref_reduce_mixed(const void *const *in, int k, const float *local, size_t rows, size_t cols, int rate,
                          void *out, size_t out_cap) {
  if (!zc2d_ref_rate_supported(rate)) return ZC2D_ERR_RATE;
  if (k < 1 || k > 16) return ZC2D_ERR_K;
  if (rows == 0 || cols == 0) return ZC2D_OK;
  if (!in || !out) return ZC2D_ERR_NULL;
  for (int c = 0; c < k; ++c)
    if (!in[c]) return ZC2D_ERR_NULL;
  if (out_cap < zc2d_ref_compressed_size(rows, cols, rate)) return ZC2D_ERR_CAPACITY;
  size_t bc = (cols + 3) / 4, br = (rows + 3) / 4;
  for (size_t bi = 0; bi < br; ++bi)
    for (size_t bj = 0; bj < bc; ++bj) {
      float s[16], f[16];
      sum_block2d(in, k, local, rows, cols, bi, bj, rate, s);
      size_t rv = rows - 4 * bi < 4 ? rows - 4 * bi : 4, cv = cols - 4 * bj < 4 ? cols - 4 * bj : 4;
      for (size_t r = 0; r < 4; ++r)
        for (size_t q = 0; q < 4; ++q) f[4 * r + q] = s[4 * (r < rv ? r : rv - 1) + (q < cv ? q : cv - 1)];
      zc2d_ref_encode_block(f, rate, (uint8_t *)out + (bi * bc + bj) * (size_t)(2 * rate));
    }
  return ZC2D_OK;
}

/* The last hop, where the sum is wanted as an fp32 matrix: nothing is re-encoded. */
int zc2d_ref_reduce_decompress(const void *const *in, int k, const float *local, size_t rows, size_t cols, int rate,
                               float *out) {
  if (!zc2d_ref_rate_supported(rate)) return ZC2D_ERR_RATE;
  if (k < 1 || k > 16) return ZC2D_ERR_K;
  if (rows == 0 || cols == 0) return ZC2D_OK;
  if (!in || !out) return ZC2D_ERR_NULL;
  for (int c = 0; c < k; ++c)
    if (!in[c]) return ZC2D_ERR_NULL;
  size_t bc = (cols + 3) / 4, br = (rows + 3) / 4;
  for (size_t bi = 0; bi < br; ++bi)
    for (size_t bj = 0; bj < bc; ++bj) {
      float s[16];
      sum_block2d(in, k, local, rows, cols, bi, bj, rate, s);
      for (size_t r = 0; r < 4; ++r)
        for (size_t q = 0; q < 4; ++q) {
          size_t rr = 4 * bi + r, cc = 4 * bj + q;
          if (rr < rows && cc < cols) out[rr * cols + cc] = s[4 * r + q];
        }
    }
  return ZC2D_OK;
}

/* ---- half-precision matrices ----------------------------------------------------------
 * bf16 / fp16 matrices (dtype codes as in zc_ref.c: 1 = bf16, 2 = fp16; the paper does not
 * state its message precision): every value is widened to fp32, which is exact, and the
 * matrix is then compressed as an fp32 matrix; decompression rounds each fp32 value to the
 * nearest half-precision value, ties to even.  The stream is the ordinary ZC-2D stream. */

int zc2d_ref_compress_half(const uint16_t *in, int dtype, size_t rows, size_t cols, int rate, void *out, size_t out_cap) {
  if (dtype != 1 && dtype != 2) return -8;
  if (!zc2d_ref_rate_supported(rate)) return ZC2D_ERR_RATE;
  if (rows == 0 || cols == 0) return ZC2D_OK;
  if (!in || !out) return ZC2D_ERR_NULL;
  if (out_cap < zc2d_ref_compressed_size(rows, cols, rate)) return ZC2D_ERR_CAPACITY;
  size_t bc = (cols + 3) / 4, br = (rows + 3) / 4;
  for (size_t bi = 0; bi < br; ++bi)
    for (size_t bj = 0; bj < bc; ++bj) {
      float x[16];
      for (int r = 0; r < 4; ++r)
        for (int c = 0; c < 4; ++c) {
          size_t rr = 4 * bi + (size_t)r, cc = 4 * bj + (size_t)c;
          if (rr >= rows) rr = rows - 1;
          if (cc >= cols) cc = cols - 1;
          x[4 * r + c] = zc_ref_widen(in[rr * cols + cc], dtype);
        }
      zc2d_ref_encode_block(x, rate, (uint8_t *)out + (bi * bc + bj) * (size_t)(2 * rate));
    }
  return ZC2D_OK;
}

int zc2d_ref_decompress_half(const void *in, size_t rows, size_t cols, int rate, int dtype, uint16_t *out) {
  if (dtype != 1 && dtype != 2) return -8;
  if (!zc2d_ref_rate_supported(rate)) return ZC2D_ERR_RATE;
  if (rows == 0 || cols == 0) return ZC2D_OK;
  if (!in || !out) return ZC2D_ERR_NULL;
  size_t bc = (cols + 3) / 4, br = (rows + 3) / 4;
  for (size_t bi = 0; bi < br; ++bi)
    for (size_t bj = 0; bj < bc; ++bj) {
      float x[16];
      zc2d_ref_decode_block((const uint8_t *)in + (bi * bc + bj) * (size_t)(2 * rate), rate, x);
      for (int r = 0; r < 4; ++r)
        for (int c = 0; c < 4; ++c) {
          size_t rr = 4 * bi + (size_t)r, cc = 4 * bj + (size_t)c;
          if (rr < rows && cc < cols) out[rr * cols + cc] = zc_ref_narrow(x[4 * r + c], dtype);
        }
    }
  return ZC2D_OK;
}
