// zc_codec.h -- per-block codec of libzc, as run by one GPU lane.
//
// One lane owns one block of 4 fp32 values.  The block's compressed form lives in
// NW = ceil(4*RATE/32) registers; nothing here touches memory except the two
// code tables, which the kernels stage in LDS.
//
// The paper names the codec family (ZFP, fixed rate; Sec. II-A, Sec. III-B) and its
// rates (Sec. IV-C, IV-F) only; the stages implemented here are: shared exponent,
// truncating block-floating-point conversion to 28 fraction bits, a five-step
// reversible lifting transform, negabinary digits, and an embedded bit-plane code
// cut at 4*RATE-8 bits behind a one-byte exponent header.
//
// How the bit-plane code is computed here (instead of bit by bit):
//   * The state of the plane coder is only n in {0..4}, the number of leading
//     coefficients already significant.  One plane's code word (at most 7 bits) is a
//     function of (n, the plane's 4 bits): an 80-entry table.  Decoding one plane is
//     a function of (n, bits left in the budget capped at 7, next 7 stream bits): a
//     5*8*128-entry table that also resolves a code word cut short by the budget.
//   * The four coefficient words are bit-transposed eight planes at a time (byte
//     gather + four masked swaps), so a plane's 4 bits are one nibble.
//   * Empty leading planes cost one zero bit each and are skipped by a count of
//     leading zeros (encoder) or trailing zeros of the payload (decoder).
//   * The stream is built by shifting code words in at the top of a register window
//     (one v_alignbit per word) and aligned once at the end.
#ifndef ZC_CODEC_H
#define ZC_CODEC_H

#include <stdint.h>

#if defined(__HIPCC__)
#define ZC_DEV __host__ __device__ __forceinline__
#else
#define ZC_DEV inline
#endif

namespace zc {

constexpr int kFractionBits = 28;

// ---- small bit helpers -------------------------------------------------------------

// ({hi,lo} >> (s & 31)) truncated to 32 bits.
ZC_DEV uint32_t alignbit(uint32_t hi, uint32_t lo, uint32_t s) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_amdgcn_alignbit(hi, lo, s);
#else
  return (uint32_t)((((uint64_t)hi << 32) | lo) >> (s & 31));
#endif
}

ZC_DEV uint32_t bitreverse(uint32_t x) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_bitreverse32(x);
#else
  x = ((x >> 1) & 0x55555555u) | ((x & 0x55555555u) << 1);
  x = ((x >> 2) & 0x33333333u) | ((x & 0x33333333u) << 2);
  x = ((x >> 4) & 0x0F0F0F0Fu) | ((x & 0x0F0F0F0Fu) << 4);
  x = ((x >> 8) & 0x00FF00FFu) | ((x & 0x00FF00FFu) << 8);
  return (x >> 16) | (x << 16);
#endif
}

ZC_DEV uint32_t count_leading_zeros(uint32_t x) { return x ? (uint32_t)__builtin_clz(x) : 32u; }
ZC_DEV uint32_t count_trailing_zeros(uint32_t x) { return x ? (uint32_t)__builtin_ctz(x) : 32u; }
ZC_DEV uint32_t umin(uint32_t a, uint32_t b) { return a < b ? a : b; }
ZC_DEV uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }

// (x & ~mask) | (y & mask)
ZC_DEV constexpr uint32_t bitselect(uint32_t mask, uint32_t y, uint32_t x) {
  return (x & ~mask) | (y & mask);
}

// Exchange, for every position p in `low` (a mask), bit p with bit p + delta.
ZC_DEV constexpr uint32_t swap_bit_groups(uint32_t x, uint32_t low, int delta) {
  return bitselect(low << delta, x << delta, bitselect(low, x >> delta, x));
}

// A 32-bit word seen as 4 rows of 8 bits (bit 8*i + m) becomes 8 rows of 4 bits
// (bit 4*m + i): four exchanges of two index bits each.
ZC_DEV constexpr uint32_t transpose_4x8(uint32_t x) {
  x = swap_bit_groups(x, 0x0000F0F0u, 12);
  x = swap_bit_groups(x, 0x00CC00CCu, 6);
  x = swap_bit_groups(x, 0x0A0A0A0Au, 3);
  x = swap_bit_groups(x, 0x22222222u, 1);
  return x;
}
ZC_DEV constexpr uint32_t transpose_8x4(uint32_t x) {
  x = swap_bit_groups(x, 0x22222222u, 1);
  x = swap_bit_groups(x, 0x0A0A0A0Au, 3);
  x = swap_bit_groups(x, 0x00CC00CCu, 6);
  x = swap_bit_groups(x, 0x0000F0F0u, 12);
  return x;
}

namespace selfcheck {
constexpr uint32_t naive_4x8(uint32_t x) {
  uint32_t y = 0;
  for (int i = 0; i < 4; ++i)
    for (int m = 0; m < 8; ++m) y |= ((x >> (8 * i + m)) & 1u) << (4 * m + i);
  return y;
}
static_assert(transpose_4x8(0x12345678u) == naive_4x8(0x12345678u), "transpose");
static_assert(transpose_4x8(0xDEADBEEFu) == naive_4x8(0xDEADBEEFu), "transpose");
static_assert(transpose_4x8(0x80000001u) == naive_4x8(0x80000001u), "transpose");
static_assert(transpose_4x8(0x0F0055AAu) == naive_4x8(0x0F0055AAu), "transpose");
static_assert(transpose_8x4(naive_4x8(0xC001D00Du)) == 0xC001D00Du, "transpose back");
static_assert(transpose_8x4(transpose_4x8(0x7E57AB1Eu)) == 0x7E57AB1Eu, "transpose back");
}  // namespace selfcheck

// ---- code tables -------------------------------------------------------------------

// One plane of the embedded code in state n (number of leading coefficients already
// significant): n verbatim bits, then group tests over the rest.  Plane bit i belongs
// to coefficient i; bit 0 of the code word is written first.
struct PlaneCode { uint32_t code; int len; int next; };

constexpr PlaneCode code_one_plane(int n, int p) {
  uint32_t code = 0;
  int len = 0;
  for (int i = 0; i < n; ++i) code |= (uint32_t)((p >> i) & 1) << len++;
  int i = n;
  while (i < 4) {
    int any = (p >> i) != 0;
    code |= (uint32_t)any << len++;
    if (!any) break;
    while (i < 3) {  // position of the first one; the last index needs no bit
      int b = (p >> i) & 1;
      code |= (uint32_t)b << len++;
      if (b) break;
      ++i;
    }
    ++i;
  }
  return PlaneCode{code, len, i};
}

// Encoder, two planes per step: entry[n*256 + (second plane << 4 | first plane)] =
// code word (<= 14 bits) | length << 14 | (byte offset of the next state's 256
// entries) << 18.
struct EncTable { uint32_t v[5 * 256]; };

constexpr EncTable build_enc_table() {
  EncTable t{};
  for (int n = 0; n <= 4; ++n)
    for (int pp = 0; pp < 256; ++pp) {
      PlaneCode a = code_one_plane(n, pp & 15);
      PlaneCode b = code_one_plane(a.next, pp >> 4);
      t.v[n * 256 + pp] = (a.code | b.code << a.len) | (uint32_t)(a.len + b.len) << 14 |
                          (uint32_t)(b.next * 256 * 4) << 18;
    }
  return t;
}

// Decoder, one plane per step: entry[(n*8 + min(bits left, 7))*128 + next 7 stream
// bits] = plane bits | bits consumed << 4 | (byte offset of the next state's 8*128
// entries) << 16.  With fewer than 7 bits left the stream bits beyond the budget are
// ignored, and a group known to hold a one that the budget cut before it was located
// gets the one at the lowest index still possible.
struct DecTable { uint32_t v[5 * 8 * 128]; };

constexpr DecTable build_dec_table() {
  DecTable t{};
  for (int n = 0; n <= 4; ++n)
    for (int avail = 0; avail < 8; ++avail)
      for (int s = 0; s < 128; ++s) {
        int left = avail, pos = 0;
        uint32_t p = 0;
        for (int i = 0; i < n && left > 0; ++i, --left) p |= (uint32_t)((s >> pos++) & 1) << i;
        int i = n;
        while (i < 4 && left > 0) {
          int any = (s >> pos++) & 1;
          --left;
          if (!any) break;
          while (i < 3 && left > 0) {
            int b = (s >> pos++) & 1;
            --left;
            if (b) break;
            ++i;
          }
          p |= 1u << i;
          ++i;
        }
        t.v[(n * 8 + avail) * 128 + s] = p | (uint32_t)pos << 4 | (uint32_t)(i * 8 * 128 * 4) << 16;
      }
  return t;
}

// ---- register window holding one compressed block ----------------------------------

template <int RATE>
struct Traits {
  static_assert(RATE >= 4 && RATE <= 32 && RATE % 4 == 0, "rate");
  static constexpr int kBlockBits = 4 * RATE;
  static constexpr int kBlockBytes = RATE / 2;
  static constexpr int kPayloadBits = 4 * RATE - 8;
  static constexpr int kWords = (4 * RATE + 31) / 32;
};

// W >>= s for s in [0, 32*NW).
template <int NW>
ZC_DEV void shift_right(uint32_t (&W)[NW], uint32_t s) {
  uint32_t bits = s & 31u, words = s >> 5;
#pragma unroll
  for (int j = 0; j < NW - 1; ++j) W[j] = alignbit(W[j + 1], W[j], bits);
  W[NW - 1] >>= bits;
  if (NW > 1) {
    uint32_t T[NW];
#pragma unroll
    for (int j = 0; j < NW; ++j) T[j] = W[j];
#pragma unroll
    for (int j = 0; j < NW; ++j) {
      uint32_t v = T[j];
#pragma unroll
      for (int d = 1; d < NW; ++d) {
        uint32_t src = 0u;
        if (j + d < NW) src = T[(j + d) % NW];
        v = (words == (uint32_t)d) ? src : v;
      }
      W[j] = v;
    }
  }
}

// Shift `len` (< 32) new bits in at the top of the window; older bits move down.
template <int NW>
ZC_DEV void shift_in(uint32_t (&W)[NW], uint32_t code, uint32_t len) {
#pragma unroll
  for (int j = 0; j < NW - 1; ++j) W[j] = alignbit(W[j + 1], W[j], len);
  W[NW - 1] = alignbit(code, W[NW - 1], len);
}

// Drop `len` (< 32) bits at the bottom of the window.
template <int NW>
ZC_DEV void shift_out(uint32_t (&W)[NW], uint32_t len) {
#pragma unroll
  for (int j = 0; j < NW - 1; ++j) W[j] = alignbit(W[j + 1], W[j], len);
  W[NW - 1] >>= len;
}

// ---- forward path ------------------------------------------------------------------

ZC_DEV float bits_to_float(uint32_t b) { return __builtin_bit_cast(float, b); }

// Four fp32 bit patterns -> biased block exponent E and the four negabinary
// coefficient words.  With m the largest magnitude as a bit pattern, E = (exponent
// field of m) + (m != 0): field + 1 for a normal maximum, 1 for a subnormal-only
// block, 0 for an all-zero block.  q_i = x_i * 2^(155 - E) truncated toward zero: the
// scaling is exact in fp32 (a result below 2^-126 may round, but truncates to 0 either
// way) and the float -> int conversion truncates.
ZC_DEV void forward_transform(const uint32_t (&x)[4], uint32_t& E, uint32_t (&u)[4]) {
  uint32_t m = umax(umax(x[0] & 0x7FFFFFFFu, x[1] & 0x7FFFFFFFu), umax(x[2] & 0x7FFFFFFFu, x[3] & 0x7FFFFFFFu));
  E = (m >> 23) + (m != 0u ? 1u : 0u);
  const int scale = 127 + kFractionBits - (int)E;
  int32_t a = (int32_t)__builtin_ldexpf(bits_to_float(x[0]), scale);
  int32_t b = (int32_t)__builtin_ldexpf(bits_to_float(x[1]), scale);
  int32_t c = (int32_t)__builtin_ldexpf(bits_to_float(x[2]), scale);
  int32_t d = (int32_t)__builtin_ldexpf(bits_to_float(x[3]), scale);
  d -= a; a += d >> 1;
  b -= c; c += b >> 1;
  c -= a; a += c >> 1;
  b -= d; d += b >> 1;
  d += b >> 2; b -= d;
  u[0] = ((uint32_t)a + 0xAAAAAAAAu) ^ 0xAAAAAAAAu;
  u[1] = ((uint32_t)b + 0xAAAAAAAAu) ^ 0xAAAAAAAAu;
  u[2] = ((uint32_t)c + 0xAAAAAAAAu) ^ 0xAAAAAAAAu;
  u[3] = ((uint32_t)d + 0xAAAAAAAAu) ^ 0xAAAAAAAAu;
}

// Byte `j` of each of four words, packed (word i -> byte i), then transposed so that
// nibble m holds bit 8*j + m of the four words.
ZC_DEV uint32_t gather_planes(const uint32_t (&r)[4], uint32_t j) {
  uint32_t g = ((r[0] >> (8 * j)) & 0xFFu) | (((r[1] >> (8 * j)) & 0xFFu) << 8) |
               (((r[2] >> (8 * j)) & 0xFFu) << 16) | (((r[3] >> (8 * j)) & 0xFFu) << 24);
  return transpose_4x8(g);
}

// Whole block: exponent byte + embedded code of the coefficients, cut at the budget.
// `enc` points at the encoder table (LDS on the GPU).  `any_lane_active(pred)` tells
// whether any lane of the wavefront still has pred set (loop control only).
template <int RATE, class AnyActive>
ZC_DEV void encode_block(const uint32_t (&x)[4], const uint32_t* enc, uint32_t (&W)[Traits<RATE>::kWords],
                         AnyActive any_lane_active) {
  constexpr int NW = Traits<RATE>::kWords;
  // every plane costs at least one bit, so at most this many planes are ever coded
  constexpr int kMaxPlanes = Traits<RATE>::kPayloadBits < 32 ? Traits<RATE>::kPayloadBits : 32;
  constexpr int kMaxSteps = (kMaxPlanes + 1) / 2;
  uint32_t E, u[4];
  forward_transform(x, E, u);
  // leading empty planes: one zero bit each
  uint32_t lead = count_leading_zeros(u[0] | u[1] | u[2] | u[3]);
  int32_t avail = Traits<RATE>::kPayloadBits - (int32_t)lead;
  uint32_t left = avail > 0 ? (uint32_t)avail : 0u;
  uint32_t r[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) r[i] = bitreverse(u[i] << (lead & 31u));  // bit t = plane (31-lead) - t; all zero if lead = 32
#pragma unroll
  for (int j = 0; j < NW; ++j) W[j] = 0;
  uint32_t state = 0;  // byte offset of the current state's table rows
  uint32_t planes = 0;
#pragma unroll 1
  for (uint32_t step = 0; step < (uint32_t)kMaxSteps; ++step) {
    if (!any_lane_active(left > 0)) break;
    if ((step & 3u) == 0u) planes = gather_planes(r, step >> 2);
    uint32_t two = (planes >> (8u * (step & 3u))) & 0xFFu;
    uint32_t e = enc[(state >> 2) + two];
    uint32_t len = umin((e >> 14) & 15u, left);
    shift_in<NW>(W, e & 0x3FFFu, len);
    left -= len;
    state = e >> 18;
  }
  // the coded bits sit at the top of the window; the first belongs at bit 8 + lead
  shift_right<NW>(W, (uint32_t)(32 * NW - Traits<RATE>::kBlockBits) + left);
  W[0] |= E;
}

// ---- inverse path ------------------------------------------------------------------

ZC_DEV void inverse_transform(const uint32_t (&u)[4], uint32_t E, float (&out)[4]) {
  int32_t a = (int32_t)((u[0] ^ 0xAAAAAAAAu) - 0xAAAAAAAAu);
  int32_t b = (int32_t)((u[1] ^ 0xAAAAAAAAu) - 0xAAAAAAAAu);
  int32_t c = (int32_t)((u[2] ^ 0xAAAAAAAAu) - 0xAAAAAAAAu);
  int32_t d = (int32_t)((u[3] ^ 0xAAAAAAAAu) - 0xAAAAAAAAu);
  // wrap-around is part of the format: unsigned adds, arithmetic shifts
  auto add = [](int32_t p, int32_t q) { return (int32_t)((uint32_t)p + (uint32_t)q); };
  auto sub = [](int32_t p, int32_t q) { return (int32_t)((uint32_t)p - (uint32_t)q); };
  b = add(b, d); d = sub(d, b >> 2);
  d = sub(d, b >> 1); b = add(b, d);
  a = sub(a, c >> 1); c = add(c, a);
  c = sub(c, b >> 1); b = add(b, c);
  a = sub(a, d >> 1); d = add(d, a);
  const int ex = (int)E - 127 - kFractionBits;
  // int -> fp32 rounds to nearest even; the scaling is exact and rounds once more only
  // for subnormal results.  A zero block arrives here with all words zero: +0.
  out[0] = __builtin_ldexpf((float)a, ex);
  out[1] = __builtin_ldexpf((float)b, ex);
  out[2] = __builtin_ldexpf((float)c, ex);
  out[3] = __builtin_ldexpf((float)d, ex);
}

// `dec` points at the decoder table.  W holds the block (bits beyond 4*RATE zero).
template <int RATE, class AnyActive>
ZC_DEV void decode_block(uint32_t (&W)[Traits<RATE>::kWords], const uint32_t* dec, float (&out)[4],
                         AnyActive any_lane_active) {
  constexpr int NW = Traits<RATE>::kWords;
  constexpr int kPayload = Traits<RATE>::kPayloadBits;
  constexpr int kMaxPlanes = kPayload < 32 ? kPayload : 32;
  const uint32_t E = W[0] & 0xFFu;
  // leading empty planes = zero bits at the start of the payload
  uint32_t lead = 0;
  {
    bool found = false;
#pragma unroll
    for (int j = 0; j < NW; ++j) {
      uint32_t w = j == 0 ? (W[0] & 0xFFFFFF00u) : W[j];
      uint32_t z = count_trailing_zeros(w);
      lead = found ? lead : lead + z;
      found = found || (w != 0);
    }
    lead -= 8u;  // the header byte
  }
  lead = umin(lead, (uint32_t)kPayload);
  uint32_t left = (uint32_t)kPayload - lead;
  // a zero block ignores its payload; after 32 empty planes nothing is left to decode
  if (E == 0u || (kPayload > 32 && lead >= 32u)) left = 0u;
  // keep the next stream bit at bit 2 of the window: bits 8..2 index the table directly
  shift_right<NW>(W, lead + 6u);
  uint32_t r[4] = {0, 0, 0, 0};
  uint32_t state = 0, planes = 0;
  uint32_t t = 0;
#pragma unroll 1
  for (; t < (uint32_t)kMaxPlanes; ++t) {
    if (!any_lane_active(left > 0)) break;
    uint32_t e = dec[((state + umin(left, 7u) * 512u) | (W[0] & 0x1FCu)) >> 2];
    uint32_t len = (e >> 4) & 7u;
    planes = alignbit(e, planes, 4);  // plane t's bits enter at the top
    shift_out<NW>(W, len);
    left -= len;
    state = e >> 16;
    if ((t & 7u) == 7u) {
      uint32_t g = transpose_8x4(planes);
#pragma unroll
      for (int i = 0; i < 4; ++i) r[i] |= ((g >> (8 * i)) & 0xFFu) << (t - 7u);
      planes = 0;
    }
  }
  if ((t & 7u) != 0u) {  // a partly filled group of planes: bring plane (t & ~7) to nibble 0
    uint32_t g = transpose_8x4(planes >> (4u * (8u - (t & 7u))));
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] |= ((g >> (8 * i)) & 0xFFu) << (t & ~7u);
  }
  uint32_t u[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) u[i] = bitreverse(r[i]) >> (lead & 31u);  // r is zero whenever lead >= 32
  inverse_transform(u, E, out);
}

}  // namespace zc
#endif  // ZC_CODEC_H
