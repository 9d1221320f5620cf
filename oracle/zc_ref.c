/*
 * zc_ref.c -- reference CPU codec for format "ZC-1".  TEST INFRASTRUCTURE ONLY.
 *
 * This is the slow, plain, single-threaded statement of what the compressed
 * collectives' codec computes.  It exists to check the GPU library; nothing in
 * the product path may call it.  It shares no code, table or constant with the
 * HIP kernels.
 *
 * What the paper fixes (Sec. II-A, Sec. III-B, Sec. IV-C/IV-F): the codec is a
 * lossy, fixed-rate compressor of the ZFP family applied to collective message
 * buffers, run at 8 bits/value for data-parallel gradients and 16 or 24
 * bits/value for tensor/pipeline/ZeRO messages; the all-reduce is a
 * reduce-scatter followed by an all-gather, both on compressed data
 * (Sec. IV-A).  The paper gives no codec internals.  The stage list
 * (block floating point -> integer lifting -> negabinary -> embedded bit-plane
 * coding cut at exactly 4*rate bits) is the one this build was asked for; every
 * constant below is a stated reading of it, listed in the design notes.
 *
 * Parity status of every function here: pinned by tests/test_oracle_*.py
 * (closed forms on IEEE bits, exhaustive round trips, brute-force search
 * decoding, hand-derived vectors, error bound, monotonicity).  Parity against
 * the ZFP library itself is NOT sought: the format differs on purpose
 * (reversible lifting, 8-bit header, 28-bit fixed point): "parity unpinned"
 * for that comparison only.
 *
 * Conventions: block = 4 consecutive fp32 values; rate R in {4,8,...,32} bits
 * per value; a block occupies exactly 4R stream bits = 8 header bits + (4R-8)
 * payload bits; stream bit t lives in bit (t mod 8) of byte t/8.
 * All integer arithmetic is 32-bit two's complement with wrap-around (build
 * with -fwrapv); >> on a signed value is an arithmetic shift.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#define ZC_REF_FRACTION_BITS 28 /* fixed-point position P */
#define ZC_REF_PLANES 32        /* bit planes of a negabinary word */

/* ---- sizes ------------------------------------------------------------- */

int zc_ref_rate_supported(int rate) {
  return rate >= 4 && rate <= 32 && (rate % 4) == 0;
}

/* ceil(n/4) blocks of 4*rate bits each; equals n*rate/8 when 4 divides n. */
size_t zc_ref_compressed_size(size_t n, int rate) {
  if (!zc_ref_rate_supported(rate)) return 0;
  size_t blocks = n / 4 + ((n % 4) ? 1 : 0);
  return blocks * (size_t)(rate / 2);
}

/* ---- stream bit access ------------------------------------------------- */

static void put_bit(uint8_t *stream, size_t t, int bit) {
  if (bit)
    stream[t >> 3] = (uint8_t)(stream[t >> 3] | (1u << (t & 7)));
  else
    stream[t >> 3] = (uint8_t)(stream[t >> 3] & ~(1u << (t & 7)));
}

static int get_bit(const uint8_t *stream, size_t t) {
  return (stream[t >> 3] >> (t & 7)) & 1;
}

/* ---- stage 1: shared exponent ------------------------------------------ */

/* Biased block exponent E.  With |x| = f * 2^eps, 1/2 <= f < 1 (the frexp
 * convention), e = max(eps over the non-zero values, -126) and E = e + 127.
 * E = 0 marks a block whose four values are all (plus or minus) zero. */
int zc_ref_block_exponent(const float x[4]) {
  int any = 0, emax = 0;
  for (int i = 0; i < 4; ++i) {
    if (x[i] != 0.0f) {
      int eps;
      (void)frexpf(x[i], &eps);
      if (!any || eps > emax) emax = eps;
      any = 1;
    }
  }
  if (!any) return 0;
  if (emax < -126) emax = -126;
  return emax + 127;
}

/* ---- stage 2: block floating point ------------------------------------- */

/* q_i = x_i * 2^(P - e), truncated toward zero.  The product is exact in
 * double (24-bit significand, exponent far inside double's range). */
void zc_ref_quantise(const float x[4], int E, int32_t q[4]) {
  int e = E - 127;
  for (int i = 0; i < 4; ++i)
    q[i] = (int32_t)trunc(ldexp((double)x[i], ZC_REF_FRACTION_BITS - e));
}

/* x_i = float(q_i) * 2^(e - P): int -> fp32 with round-to-nearest-even, then
 * an IEEE scaling by a power of two (rounds again only for subnormal results). */
void zc_ref_dequantise(const int32_t q[4], int E, float x[4]) {
  int e = E - 127;
  for (int i = 0; i < 4; ++i)
    x[i] = ldexpf((float)q[i], e - ZC_REF_FRACTION_BITS);
}

/* ---- stage 3: reversible lifting transform ------------------------------ */

/* Five lifting steps; each adds to one lane a function of another lane, so
 * each is undone exactly by subtracting the same quantity.  Output order is
 * (mean, linear, quadratic, cubic). */
void zc_ref_fwd_lift(int32_t v[4]) {
  int32_t a = v[0], b = v[1], c = v[2], d = v[3];
  d -= a; a += d >> 1;
  b -= c; c += b >> 1;
  c -= a; a += c >> 1;
  b -= d; d += b >> 1;
  d += b >> 2; b -= d;
  v[0] = a; v[1] = b; v[2] = c; v[3] = d;
}

void zc_ref_inv_lift(int32_t v[4]) {
  int32_t a = v[0], b = v[1], c = v[2], d = v[3];
  b += d; d -= b >> 2;
  d -= b >> 1; b += d;
  a -= c >> 1; c += a;
  c -= b >> 1; b += c;
  a -= d >> 1; d += a;
  v[0] = a; v[1] = b; v[2] = c; v[3] = d;
}

/* ---- stage 4: negabinary ------------------------------------------------ */

/* u has the digits of c in base -2: c = sum_k bit_k(u) * (-2)^k. */
uint32_t zc_ref_negabinary(int32_t c) {
  return ((uint32_t)c + 0xAAAAAAAAu) ^ 0xAAAAAAAAu;
}

int32_t zc_ref_inv_negabinary(uint32_t u) {
  return (int32_t)((u ^ 0xAAAAAAAAu) - 0xAAAAAAAAu);
}

/* ---- stage 5: embedded bit-plane coder ---------------------------------- */

/* Writes at most `budget` bits, one per element of bits[] (values 0/1), most
 * significant plane first.  Elements never written are set to 0.  Returns the
 * number of bits written. */
int zc_ref_encode_planes(const uint32_t u[4], int budget, uint8_t *bits) {
  int left = budget, w = 0;
  int n = 0; /* leading coefficients already known to be significant */
  for (int t = 0; t < budget; ++t) bits[t] = 0;
  for (int k = ZC_REF_PLANES - 1; k >= 0 && left > 0; --k) {
    int p[4];
    for (int i = 0; i < 4; ++i) p[i] = (u[i] >> k) & 1;
    /* (i) verbatim bits of the significant coefficients */
    for (int i = 0; i < n && left > 0; ++i) { bits[w++] = (uint8_t)p[i]; --left; }
    /* (ii) group tests over the remaining coefficients */
    int i = n;
    while (i < 4 && left > 0) {
      int g = 0;
      for (int j = i; j < 4; ++j) g |= p[j];
      bits[w++] = (uint8_t)g; --left;
      if (!g) break;
      /* locate the first one; at index 3 it is implied */
      while (i < 3 && left > 0) {
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

/* Mirror of the encoder.  Bits beyond the budget are never read. */
void zc_ref_decode_planes(const uint8_t *bits, int budget, uint32_t u[4]) {
  int left = budget, r = 0;
  int n = 0;
  u[0] = u[1] = u[2] = u[3] = 0;
  for (int k = ZC_REF_PLANES - 1; k >= 0 && left > 0; --k) {
    for (int i = 0; i < n && left > 0; ++i) {
      if (bits[r++]) u[i] |= 1u << k;
      --left;
    }
    int i = n;
    while (i < 4 && left > 0) {
      int g = bits[r++]; --left;
      if (!g) break;
      while (i < 3 && left > 0) {
        int b = bits[r++]; --left;
        if (b) break;
        ++i;
      }
      /* the group holds a one: it sits at i, the smallest index still
       * possible (also when the budget ended before it was located) */
      u[i] |= 1u << k;
      ++i;
    }
    n = i;
  }
}

/* ---- one block ---------------------------------------------------------- */

static void encode_block(const float x[4], int rate, uint8_t *stream, size_t bit0) {
  const int B = 4 * rate, budget = B - 8;
  for (int t = 0; t < B; ++t) put_bit(stream, bit0 + (size_t)t, 0);
  int E = zc_ref_block_exponent(x);
  if (E == 0) return; /* zero block: all 4R bits are zero */
  for (int t = 0; t < 8; ++t) put_bit(stream, bit0 + (size_t)t, (E >> t) & 1);
  int32_t q[4];
  zc_ref_quantise(x, E, q);
  zc_ref_fwd_lift(q);
  uint32_t u[4];
  for (int i = 0; i < 4; ++i) u[i] = zc_ref_negabinary(q[i]);
  uint8_t bits[4 * 32 - 8];
  zc_ref_encode_planes(u, budget, bits);
  for (int t = 0; t < budget; ++t) put_bit(stream, bit0 + 8 + (size_t)t, bits[t]);
}

static void decode_block(const uint8_t *stream, size_t bit0, int rate, float x[4]) {
  const int budget = 4 * rate - 8;
  int E = 0;
  for (int t = 0; t < 8; ++t) E |= get_bit(stream, bit0 + (size_t)t) << t;
  if (E == 0) { x[0] = x[1] = x[2] = x[3] = 0.0f; return; }
  uint8_t bits[4 * 32 - 8];
  for (int t = 0; t < budget; ++t) bits[t] = (uint8_t)get_bit(stream, bit0 + 8 + (size_t)t);
  uint32_t u[4];
  zc_ref_decode_planes(bits, budget, u);
  int32_t c[4];
  for (int i = 0; i < 4; ++i) c[i] = zc_ref_inv_negabinary(u[i]);
  zc_ref_inv_lift(c);
  zc_ref_dequantise(c, E, x);
}

/* Single-block entry points for tests. */
void zc_ref_encode_block(const float x[4], int rate, uint8_t *out /* rate/2 bytes */) {
  encode_block(x, rate, out, 0);
}
void zc_ref_decode_block(const uint8_t *in, int rate, float x[4]) {
  decode_block(in, 0, rate, x);
}

/* ---- whole buffers (host pointers) -------------------------------------- */

enum { ZC_REF_OK = 0, ZC_REF_ERR_NULL = -1, ZC_REF_ERR_RATE = -2,
       ZC_REF_ERR_CAPACITY = -4, ZC_REF_ERR_K = -5 };

/* A ragged last block repeats the last valid value in its unused lanes. */
static void load_block(const float *in, size_t n, size_t j, float x[4]) {
  for (int i = 0; i < 4; ++i) {
    size_t idx = 4 * j + (size_t)i;
    x[i] = in[idx < n ? idx : n - 1];
  }
}

int zc_ref_compress(const float *in, size_t n, int rate, void *out, size_t out_cap) {
  if (!zc_ref_rate_supported(rate)) return ZC_REF_ERR_RATE;
  if (n == 0) return ZC_REF_OK;
  if (!in || !out) return ZC_REF_ERR_NULL;
  if (out_cap < zc_ref_compressed_size(n, rate)) return ZC_REF_ERR_CAPACITY;
  size_t blocks = (n + 3) / 4;
  for (size_t j = 0; j < blocks; ++j) {
    float x[4];
    load_block(in, n, j, x);
    encode_block(x, rate, (uint8_t *)out, j * (size_t)(4 * rate));
  }
  return ZC_REF_OK;
}

int zc_ref_decompress(const void *in, size_t n, int rate, float *out) {
  if (!zc_ref_rate_supported(rate)) return ZC_REF_ERR_RATE;
  if (n == 0) return ZC_REF_OK;
  if (!in || !out) return ZC_REF_ERR_NULL;
  size_t blocks = (n + 3) / 4;
  for (size_t j = 0; j < blocks; ++j) {
    float x[4];
    decode_block((const uint8_t *)in, j * (size_t)(4 * rate), rate, x);
    for (int i = 0; i < 4; ++i)
      if (4 * j + (size_t)i < n) out[4 * j + (size_t)i] = x[i];
  }
  return ZC_REF_OK;
}

/* The step a rank performs inside a compressed reduce-scatter (Sec. IV-A):
 * decode the k incoming chunks, add them element by element in fp32 in index
 * order ((d0 + d1) + d2) + ..., and encode the sum (new shared exponents).
 * `out` may be the same buffer as in[0]. */
int zc_ref_reduce_compressed(const void *const *in, int k, size_t n, int rate,
                             void *out, size_t out_cap) {
  if (!zc_ref_rate_supported(rate)) return ZC_REF_ERR_RATE;
  if (k < 1 || k > 16) return ZC_REF_ERR_K;
  if (n == 0) return ZC_REF_OK;
  if (!in || !out) return ZC_REF_ERR_NULL;
  for (int c = 0; c < k; ++c)
    if (!in[c]) return ZC_REF_ERR_NULL;
  if (out_cap < zc_ref_compressed_size(n, rate)) return ZC_REF_ERR_CAPACITY;
  size_t blocks = (n + 3) / 4;
  for (size_t j = 0; j < blocks; ++j) {
    size_t bit0 = j * (size_t)(4 * rate);
    float s[4], d[4];
    decode_block((const uint8_t *)in[0], bit0, rate, s);
    for (int c = 1; c < k; ++c) {
      decode_block((const uint8_t *)in[c], bit0, rate, d);
      for (int i = 0; i < 4; ++i) {
        volatile float t = s[i] + d[i]; /* one fp32 rounding per add */
        s[i] = t;
      }
    }
    /* the result is compress(sum): a ragged last block is padded with the
     * last valid sum, not with the sum of the inputs' pad lanes */
    for (int i = 0; i < 4; ++i)
      if (4 * j + (size_t)i >= n) s[i] = s[(n - 1) - 4 * j];
    encode_block(s, rate, (uint8_t *)out, bit0);
  }
  return ZC_REF_OK;
}

/* ---- ring-hop variants of the reduce step -------------------------------- */

/* Sum of block j over the k chunks and, if `local` is given, the raw local
 * values added last: ((d0 + d1) + ... + d_{k-1}) + x.  Lanes beyond n take
 * the local pad rule (last valid value repeated) before the add; they are
 * replaced by the caller anyway. */
static void sum_block(const void *const *in, int k, const float *local, size_t n, size_t j,
                      int rate, float s[4]) {
  size_t bit0 = j * (size_t)(4 * rate);
  float d[4];
  if (k > 0) {
    decode_block((const uint8_t *)in[0], bit0, rate, s);
  } else {
    s[0] = s[1] = s[2] = s[3] = 0.0f;
  }
  for (int c = 1; c < k; ++c) {
    decode_block((const uint8_t *)in[c], bit0, rate, d);
    for (int i = 0; i < 4; ++i) {
      volatile float t = s[i] + d[i];
      s[i] = t;
    }
  }
  if (local) {
    load_block(local, n, j, d);
    for (int i = 0; i < 4; ++i) {
      volatile float t = s[i] + d[i];
      s[i] = t;
    }
  }
}

/* A ring hop whose local contribution is still raw fp32 (Sec. IV-A: each
 * rank adds its own gradients to what it received before forwarding):
 * out = compress(((d0 + ... + d_{k-1}) + local)).  k >= 1; local may be NULL,
 * which makes this zc_ref_reduce_compressed. */
int zc_ref_reduce_mixed(const void *const *in, int k, const float *local, size_t n, int rate,
                        void *out, size_t out_cap) {
  if (!zc_ref_rate_supported(rate)) return ZC_REF_ERR_RATE;
  if (k < 1 || k > 16) return ZC_REF_ERR_K;
  if (n == 0) return ZC_REF_OK;
  if (!in || !out) return ZC_REF_ERR_NULL;
  for (int c = 0; c < k; ++c)
    if (!in[c]) return ZC_REF_ERR_NULL;
  if (out_cap < zc_ref_compressed_size(n, rate)) return ZC_REF_ERR_CAPACITY;
  size_t blocks = (n + 3) / 4;
  for (size_t j = 0; j < blocks; ++j) {
    float s[4];
    sum_block(in, k, local, n, j, rate, s);
    for (int i = 0; i < 4; ++i)
      if (4 * j + (size_t)i >= n) s[i] = s[(n - 1) - 4 * j];
    encode_block(s, rate, (uint8_t *)out, j * (size_t)(4 * rate));
  }
  return ZC_REF_OK;
}

/* The last hop, where the sum is wanted as fp32: out[i] = ((d0 + ... +
 * d_{k-1}) + local)[i], nothing re-encoded.  local may be NULL. */
int zc_ref_reduce_decompress(const void *const *in, int k, const float *local, size_t n, int rate,
                             float *out) {
  if (!zc_ref_rate_supported(rate)) return ZC_REF_ERR_RATE;
  if (k < 1 || k > 16) return ZC_REF_ERR_K;
  if (n == 0) return ZC_REF_OK;
  if (!in || !out) return ZC_REF_ERR_NULL;
  for (int c = 0; c < k; ++c)
    if (!in[c]) return ZC_REF_ERR_NULL;
  size_t blocks = (n + 3) / 4;
  for (size_t j = 0; j < blocks; ++j) {
    float s[4];
    sum_block(in, k, local, n, j, rate, s);
    for (int i = 0; i < 4; ++i)
      if (4 * j + (size_t)i < n) out[4 * j + (size_t)i] = s[i];
  }
  return ZC_REF_OK;
}

/* ---- half-precision messages ---------------------------------------------- */
/* The paper does not state the precision of its messages; LLM training traffic
 * is commonly bf16 or fp16.  These entry points run the same codec on such
 * buffers: every value is widened to fp32 exactly before compression (both
 * formats are subsets of fp32), and decompressed values are narrowed with
 * round-to-nearest-even.  The stream format is unchanged. */

enum { ZC_REF_F32 = 0, ZC_REF_BF16 = 1, ZC_REF_F16 = 2 };

/* bf16 is the upper half of an fp32. */
static float widen_bf16(uint16_t h) {
  uint32_t b = (uint32_t)h << 16;
  float f;
  memcpy(&f, &b, 4);
  return f;
}

/* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
static float widen_f16(uint16_t h) {
  int sign = (h >> 15) & 1, ex = (h >> 10) & 31, frac = h & 1023;
  float v;
  if (ex == 0) v = ldexpf((float)frac, -24);                /* zero and subnormals */
  else if (ex == 31) v = frac ? NAN : INFINITY;
  else v = ldexpf((float)(frac | 1024), ex - 25);
  return sign ? -v : v;
}

float zc_ref_widen(uint16_t h, int dtype) { return dtype == ZC_REF_BF16 ? widen_bf16(h) : widen_f16(h); }

/* Nearest representable value, ties to the even fraction; magnitudes beyond
 * the largest finite value round to infinity as IEEE prescribes. */
uint16_t zc_ref_narrow(float f, int dtype) {
  if (f != f) return dtype == ZC_REF_BF16 ? 0x7FC0 : 0x7E00;
  uint16_t sign = signbit(f) ? 0x8000 : 0;
  double a = fabs((double)f);
  int frac_bits = dtype == ZC_REF_BF16 ? 7 : 10;
  int emin = dtype == ZC_REF_BF16 ? -126 : -14;   /* exponent of the smallest normal */
  int emax = dtype == ZC_REF_BF16 ? 127 : 15;
  int exp_bits_max = dtype == ZC_REF_BF16 ? 255 : 31;
  if (a == 0.0) return sign;
  if (isinf(a)) return (uint16_t)(sign | (exp_bits_max << frac_bits));
  int e;
  (void)frexp(a, &e);            /* a = m * 2^e, 0.5 <= m < 1 */
  e -= 1;                        /* a = m' * 2^e, 1 <= m' < 2 */
  if (e < emin) e = emin;        /* subnormal range: fixed quantum */
  double q = ldexp(a, frac_bits - e);       /* in units of the last fraction bit: exact */
  double r = nearbyint(q);                  /* round to nearest, ties to even (default mode) */
  /* r is in [2^frac_bits, 2^(frac_bits+1)] for normals, [0, 2^frac_bits] for subnormals */
  long long units = (long long)r;
  long long biased;
  if (units >> (frac_bits + 1)) { units >>= 1; e += 1; }    /* rounded up to the next power of two */
  if (units >> frac_bits) biased = ((long long)(e - emin + 1) << frac_bits) + (units - (1LL << frac_bits));
  else biased = units;                                      /* subnormal or zero */
  if (e > emax) biased = (long long)exp_bits_max << frac_bits; /* overflow -> infinity */
  return (uint16_t)(sign | (uint16_t)biased);
}

int zc_ref_compress_half(const uint16_t *in, int dtype, size_t n, int rate, void *out, size_t out_cap) {
  if (dtype != ZC_REF_BF16 && dtype != ZC_REF_F16) return -8;
  if (!zc_ref_rate_supported(rate)) return ZC_REF_ERR_RATE;
  if (n == 0) return ZC_REF_OK;
  if (!in || !out) return ZC_REF_ERR_NULL;
  if (out_cap < zc_ref_compressed_size(n, rate)) return ZC_REF_ERR_CAPACITY;
  size_t blocks = (n + 3) / 4;
  for (size_t j = 0; j < blocks; ++j) {
    float x[4];
    for (int i = 0; i < 4; ++i) {
      size_t idx = 4 * j + (size_t)i;
      x[i] = zc_ref_widen(in[idx < n ? idx : n - 1], dtype);
    }
    encode_block(x, rate, (uint8_t *)out, j * (size_t)(4 * rate));
  }
  return ZC_REF_OK;
}

int zc_ref_decompress_half(const void *in, size_t n, int rate, int dtype, uint16_t *out) {
  if (dtype != ZC_REF_BF16 && dtype != ZC_REF_F16) return -8;
  if (!zc_ref_rate_supported(rate)) return ZC_REF_ERR_RATE;
  if (n == 0) return ZC_REF_OK;
  if (!in || !out) return ZC_REF_ERR_NULL;
  size_t blocks = (n + 3) / 4;
  for (size_t j = 0; j < blocks; ++j) {
    float x[4];
    decode_block((const uint8_t *)in, j * (size_t)(4 * rate), rate, x);
    for (int i = 0; i < 4; ++i)
      if (4 * j + (size_t)i < n) out[4 * j + (size_t)i] = zc_ref_narrow(x[i], dtype);
  }
  return ZC_REF_OK;
}

