/*
 * zl_ref.c -- reference CPU codec for the lossless format "ZL-1".  TEST INFRASTRUCTURE ONLY.
 *
 * The paper's first hybrid scheme sends model-parallel traffic through a lossless
 * GPU codec of the MPC kind, which it describes only as exploiting the similarity of
 * consecutive floating-point values (Sec. II-A, Sec. III-A with its table of
 * collectives).  It gives no format.  What is built here is a format of that kind,
 * stated in full below: describe each 32-bit word of a group of 32 nearby words by its
 * distance from the group's largest magnitude, bit-transpose the 32 residuals, and drop
 * the transposed words that are zero (values of similar magnitude share their upper
 * exponent bits, half-precision content its empty lower half, a smooth series nearly
 * everything).  Every choice is a reading listed in the design notes.  Nothing here is
 * shared with the HIP kernels.
 *
 * Format.  The message is n 32-bit words (fp32 bit patterns; the codec never
 * interprets them, so NaN and infinities are as good as any other pattern).
 *
 *   chunk      8192 consecutive words; the last chunk is filled up with zero words.
 *   group      a chunk is 256 groups of 32 words: word j of group g is the chunk's
 *              word 1024*(j/4) + 4*g + (j%4)  (four consecutive words, then a stride
 *              of 1024: the order in which 256 lanes read 16 bytes each).
 *   reference  m[g] = the largest of w[g][j] & 0x7FFFFFFF over the group (for floats: the
 *              largest magnitude, as a bit pattern).
 *   residual   r[g][j] = (w[g][j] & 0x80000000) | (m[g] - (w[g][j] & 0x7FFFFFFF)):
 *              the sign bit as it is, below it the distance from the reference.
 *   plane      p[g][k], k = 0..31: bit j of p[g][k] = bit k of r[g][j].
 *   bitmap     b[g]: bit k set iff p[g][k] != 0.
 *
 *   stream     header (32 bytes) | table (8 bytes per chunk) | payload
 *   header     u32 magic 0x31304C5A ("ZL01"), u32 number of chunks, u64 n,
 *              u64 total bytes of the stream, u64 zero
 *   table      entry c: bits 63..62 = binary 10, bits 61..0 = byte offset, from the
 *              start of the payload, at which chunk c ends (chunk c starts where
 *              chunk c-1 ends, chunk 0 at 0)
 *   chunk      the 256 references m[0..255], the 256 bitmaps b[0..255] (u32 each), then
 *              for g = 0..255 the non-zero planes p[g][k] in ascending k (u32 each)
 * All integers little-endian.  n = 0 gives the header alone.
 *
 * Parity status: pinned by tests/test_oracle_lossless.py.
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#define ZL_MAGIC 0x31304C5Au
#define ZL_CHUNK_WORDS 8192u
#define ZL_GROUPS 256u
#define ZL_HEADER_BYTES 32u
#define ZL_ENTRY_DONE ((uint64_t)2 << 62)
#define ZL_OFFSET_MASK (((uint64_t)1 << 62) - 1)

enum { ZL_OK = 0, ZL_ERR_NULL = -1, ZL_ERR_SIZE = -3, ZL_ERR_CAPACITY = -4, ZL_ERR_STREAM = -9 };

/* ---- the pieces ------------------------------------------------------------- */

/* Index within its chunk of word j of group g. */
uint32_t zl_ref_word_index(uint32_t g, uint32_t j) { return 1024u * (j / 4u) + 4u * g + (j % 4u); }

/* Reference of a group and its residuals. */
uint32_t zl_ref_residuals(const uint32_t w[32], uint32_t r[32]) {
  uint32_t m = 0;
  for (int j = 0; j < 32; ++j)
    if ((w[j] & 0x7FFFFFFFu) > m) m = w[j] & 0x7FFFFFFFu;
  for (int j = 0; j < 32; ++j) r[j] = (w[j] & 0x80000000u) | (m - (w[j] & 0x7FFFFFFFu));
  return m;
}

/* Words from reference and residuals.  A stream may hold residuals that no encoder
 * produces (distance larger than the reference): the subtraction then wraps within 31
 * bits, so that every stream decodes to something. */
void zl_ref_words(uint32_t m, const uint32_t r[32], uint32_t w[32]) {
  for (int j = 0; j < 32; ++j) w[j] = (r[j] & 0x80000000u) | ((m - (r[j] & 0x7FFFFFFFu)) & 0x7FFFFFFFu);
}

void zl_ref_planes(const uint32_t r[32], uint32_t p[32]) {
  for (int k = 0; k < 32; ++k) {
    uint32_t v = 0;
    for (int j = 0; j < 32; ++j) v |= ((r[j] >> k) & 1u) << j;
    p[k] = v;
  }
}

void zl_ref_unplanes(const uint32_t p[32], uint32_t r[32]) {
  for (int j = 0; j < 32; ++j) {
    uint32_t v = 0;
    for (int k = 0; k < 32; ++k) v |= ((p[k] >> j) & 1u) << k;
    r[j] = v;
  }
}

size_t zl_ref_chunks(size_t n) { return (n + ZL_CHUNK_WORDS - 1) / ZL_CHUNK_WORDS; }

/* Largest stream n words can produce: every plane of every group non-zero. */
size_t zl_ref_max_compressed_size(size_t n) {
  return ZL_HEADER_BYTES + zl_ref_chunks(n) * (8u + 8u * ZL_GROUPS + 4u * ZL_CHUNK_WORDS);
}

/* ---- little-endian stores and loads ------------------------------------------------ */

static void put32(uint8_t *p, uint32_t v) { for (int i = 0; i < 4; ++i) p[i] = (uint8_t)(v >> (8 * i)); }
static void put64(uint8_t *p, uint64_t v) { for (int i = 0; i < 8; ++i) p[i] = (uint8_t)(v >> (8 * i)); }
static uint32_t get32(const uint8_t *p) { uint32_t v = 0; for (int i = 0; i < 4; ++i) v |= (uint32_t)p[i] << (8 * i); return v; }
static uint64_t get64(const uint8_t *p) { uint64_t v = 0; for (int i = 0; i < 8; ++i) v |= (uint64_t)p[i] << (8 * i); return v; }

/* ---- whole messages (host pointers) ------------------------------------------------ */

int zl_ref_compress(const uint32_t *in, size_t n, void *out, size_t out_cap, size_t *out_bytes) {
  if (!out || !out_bytes || (n && !in)) return ZL_ERR_NULL;
  if (out_cap < zl_ref_max_compressed_size(n)) return ZL_ERR_CAPACITY;
  uint8_t *s = (uint8_t *)out;
  size_t chunks = zl_ref_chunks(n);
  if (chunks > 0xFFFFFFFFu) return ZL_ERR_SIZE;
  uint8_t *table = s + ZL_HEADER_BYTES, *payload = table + 8 * chunks;
  uint64_t end = 0;
  for (size_t c = 0; c < chunks; ++c) {
    uint8_t *refs = payload + end, *bitmaps = refs + 4 * ZL_GROUPS, *words = bitmaps + 4 * ZL_GROUPS;
    for (uint32_t g = 0; g < ZL_GROUPS; ++g) {
      uint32_t w[32], r[32], p[32], b = 0;
      for (uint32_t j = 0; j < 32; ++j) {
        size_t i = c * ZL_CHUNK_WORDS + zl_ref_word_index(g, j);
        w[j] = i < n ? in[i] : 0u;
      }
      put32(refs + 4 * g, zl_ref_residuals(w, r));
      zl_ref_planes(r, p);
      for (int k = 0; k < 32; ++k)
        if (p[k]) { b |= 1u << k; put32(words, p[k]); words += 4; }
      put32(bitmaps + 4 * g, b);
    }
    end = (uint64_t)(words - payload);
    put64(table + 8 * c, ZL_ENTRY_DONE | end);
  }
  uint64_t total = ZL_HEADER_BYTES + 8 * (uint64_t)chunks + end;
  put32(s, ZL_MAGIC);
  put32(s + 4, (uint32_t)chunks);
  put64(s + 8, (uint64_t)n);
  put64(s + 16, total);
  put64(s + 24, 0);
  *out_bytes = (size_t)total;
  return ZL_OK;
}

/* Total bytes of a stream, from its header; 0 if the header is not one. */
size_t zl_ref_stream_bytes(const void *in, size_t in_bytes) {
  const uint8_t *s = (const uint8_t *)in;
  if (!s || in_bytes < ZL_HEADER_BYTES || get32(s) != ZL_MAGIC) return 0;
  return (size_t)get64(s + 16);
}

int zl_ref_decompress(const void *in, size_t in_bytes, size_t n, uint32_t *out) {
  if (!in || (n && !out)) return ZL_ERR_NULL;
  const uint8_t *s = (const uint8_t *)in;
  if (in_bytes < ZL_HEADER_BYTES || get32(s) != ZL_MAGIC) return ZL_ERR_STREAM;
  size_t chunks = zl_ref_chunks(n);
  if (get64(s + 8) != (uint64_t)n || get32(s + 4) != (uint32_t)chunks) return ZL_ERR_STREAM;
  uint64_t total = get64(s + 16);
  if (total > in_bytes || total < ZL_HEADER_BYTES + 8 * (uint64_t)chunks) return ZL_ERR_STREAM;
  const uint8_t *table = s + ZL_HEADER_BYTES, *payload = table + 8 * chunks;
  uint64_t room = total - ZL_HEADER_BYTES - 8 * (uint64_t)chunks, start = 0;
  for (size_t c = 0; c < chunks; ++c) {
    uint64_t e = get64(table + 8 * c);
    uint64_t end = e & ZL_OFFSET_MASK;
    if ((e >> 62) != 2 || end > room || end < start + 8 * ZL_GROUPS) return ZL_ERR_STREAM;
    const uint8_t *refs = payload + start, *bitmaps = refs + 4 * ZL_GROUPS, *words = bitmaps + 4 * ZL_GROUPS;
    for (uint32_t g = 0; g < ZL_GROUPS; ++g) {
      uint32_t b = get32(bitmaps + 4 * g), p[32], r[32], w[32];
      for (int k = 0; k < 32; ++k) {
        p[k] = 0;
        if ((b >> k) & 1u) {
          if ((uint64_t)(words - payload) + 4 > end) return ZL_ERR_STREAM;
          p[k] = get32(words);
          words += 4;
        }
      }
      zl_ref_unplanes(p, r);
      zl_ref_words(get32(refs + 4 * g), r, w);
      for (uint32_t j = 0; j < 32; ++j) {
        size_t i = c * ZL_CHUNK_WORDS + zl_ref_word_index(g, j);
        if (i < n) out[i] = w[j];
      }
    }
    if ((uint64_t)(words - payload) != end) return ZL_ERR_STREAM;
    start = end;
  }
  return ZL_OK;
}

/* ---- 16-bit messages ------------------------------------------------------------------
 * Half-precision traffic (bf16 or fp16; the paper does not say what its messages hold)
 * goes through the same format: the message of n 16-bit words v is coded as the n 32-bit
 * words v << 16.  For bf16 that is the value widened to fp32; for any content it is a
 * plain embedding, so every pattern comes back.  The empty lower halves cost nothing in
 * the stream (their planes are zero). */

int zl_ref_compress16(const uint16_t *in, size_t n, void *out, size_t out_cap, size_t *out_bytes,
                      uint32_t *work /* n words */) {
  if (n && (!in || !work)) return ZL_ERR_NULL;
  for (size_t i = 0; i < n; ++i) work[i] = (uint32_t)in[i] << 16;
  return zl_ref_compress(work, n, out, out_cap, out_bytes);
}

/* The upper halves of the decoded words (for a stream made by zl_ref_compress16 the lower
 * halves are zero). */
int zl_ref_decompress16(const void *in, size_t in_bytes, size_t n, uint16_t *out, uint32_t *work /* n words */) {
  if (n && (!out || !work)) return ZL_ERR_NULL;
  int rc = zl_ref_decompress(in, in_bytes, n, work);
  if (rc != ZL_OK) return rc;
  for (size_t i = 0; i < n; ++i) out[i] = (uint16_t)(work[i] >> 16);
  return ZL_OK;
}
