// zc_codec.h -- per-block codec of libzc, as run by one GPU lane.
//
// One lane owns one block of 4 fp32 values.  The block's compressed form lives in
// NW = ceil(4*RATE/32) registers; nothing here touches memory except the code
// tables, which the kernels stage in LDS.
//
// The paper names the codec family (ZFP, fixed rate; Sec. II-A, Sec. III-B) and its
// rates (Sec. IV-C, IV-F) only; the stages implemented here are: shared exponent,
// truncating block-floating-point conversion to 28 fraction bits, a five-step
// reversible lifting transform, negabinary digits, and an embedded bit-plane code
// cut at 4*RATE-8 bits behind a one-byte exponent header.
//
// How the bit-plane code is computed here (instead of bit by bit):
//   * The state of the plane coder is only n in {0..4}, the number of leading
//     coefficients already significant, and from n = 3 on a plane is coded as its four
//     bits as they are.  So both coders walk their tables only until every lane of the
//     wavefront has three significant coefficients (or no budget left) and handle the
//     rest of the block as a literal string of planes, without a loop (see encode_block
//     and decode_block).
//   * Encoder table: (n, two planes as a byte of the literal string) -> code word of at
//     most 14 bits, its length and the next state.  Decoder tables: (n, next 9 stream
//     bits) -> one or two planes, bits used, next state, while the budget cannot cut
//     what is read; (n, bits left capped at 7, that many stream bits) -> one plane near
//     the budget's end, which also resolves a code word cut short by the budget.  At
//     rate 4 the payload is a single byte: one 8192-entry table encodes it and one
//     256-entry table holds the decoded block up to its power-of-two scale.
//   * Decoded plane bits are collected in four byte lanes, one per coefficient, so no bit
//     transposition is needed; literal planes go through 256-entry spread / pair tables.
//   * Empty leading planes cost one zero bit each and are skipped by a count of
//     leading zeros (encoder) or trailing zeros of the payload (decoder).
//   * The stream is built by shifting code words in at the top of a register window
//     (one v_alignbit per word) and put in place by one funnel shift at the end.
#ifndef ZC_CODEC_H
#define ZC_CODEC_H

#include <stddef.h>
#include <stdint.h>

#if defined(__HIPCC__)
#define ZC_DEV __host__ __device__ __forceinline__
#else
#define ZC_DEV inline
#endif

namespace zc {

constexpr int kFractionBits = 28;

// ---- small bit helpers -------------------------------------------------------------

// Makes v opaque to the compiler at this point: it is computed once, as a whole, and what
// follows starts from that register.  (Without it the compiler may split a computation by the
// bits each later use needs and do much of it twice.)
ZC_DEV void materialise(uint32_t& v) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm("" : "+v"(v));
#else
  (void)v;
#endif
}

// ({hi,lo} >> (s & 31)) truncated to 32 bits.
ZC_DEV uint32_t alignbit(uint32_t hi, uint32_t lo, uint32_t s) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_amdgcn_alignbit(hi, lo, s);
#else
  return (uint32_t)((((uint64_t)hi << 32) | lo) >> (s & 31));
#endif
}

// Byte j of the result is byte sel[j] of the eight bytes {hi, lo} (0..3 = lo, 4..7 = hi);
// a selector byte of 0x0c gives a zero byte.
ZC_DEV uint32_t permute_bytes(uint32_t hi, uint32_t lo, uint32_t sel) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_amdgcn_perm(hi, lo, sel);
#else
  const uint64_t pool = ((uint64_t)hi << 32) | lo;
  uint32_t r = 0;
  for (int j = 0; j < 4; ++j) {
    const uint32_t c = (sel >> (8 * j)) & 0xFFu;
    const uint32_t b = c < 8u ? (uint32_t)(pool >> (8u * c)) & 0xFFu : 0u;
    r |= b << (8 * j);
  }
  return r;
#endif
}

ZC_DEV uint32_t count_leading_zeros(uint32_t x) { return x ? (uint32_t)__builtin_clz(x) : 32u; }
// The same for x != 0; for x = 0 a value that callers may only use as a shift count for
// zero words (the instruction gives -1 there, and the test for zero is saved).
ZC_DEV uint32_t count_leading_zeros_nonzero(uint32_t x) {
#if defined(__HIP_DEVICE_COMPILE__)
  uint32_t r;
  asm("v_ffbh_u32 %0, %1" : "=v"(r) : "v"(x));
  return r;
#else
  return x ? (uint32_t)__builtin_clz(x) : 0xFFFFFFFFu;
#endif
}
ZC_DEV uint32_t count_trailing_zeros(uint32_t x) { return x ? (uint32_t)__builtin_ctz(x) : 32u; }
ZC_DEV uint32_t umin(uint32_t a, uint32_t b) { return a < b ? a : b; }
ZC_DEV uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }
ZC_DEV float bits_to_float(uint32_t b) { return __builtin_bit_cast(float, b); }

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

// The reverse: read one plane in state n from the low bits of `s`, of which only
// `avail` are inside the budget.  A group known to hold a one that the budget cut
// before it was located gets the one at the lowest index still possible.
struct PlaneBits { uint32_t p; int used; int next; };

constexpr PlaneBits read_one_plane(int n, int avail, uint32_t s) {
  int left = avail, pos = 0;
  uint32_t p = 0;
  for (int i = 0; i < n && left > 0; ++i, --left) p |= ((s >> pos++) & 1u) << i;
  int i = n;
  while (i < 4 && left > 0) {
    int any = (int)((s >> pos++) & 1u);
    --left;
    if (!any) break;
    while (i < 3 && left > 0) {
      int b = (int)((s >> pos++) & 1u);
      --left;
      if (b) break;
      ++i;
    }
    p |= 1u << i;
    ++i;
  }
  return PlaneBits{p, pos, i};
}

// Encoder, two planes per step.  Index = n*256 + x, where the low four bits of x are the
// earlier plane and the high four bits the later one, bit i of each belonging to coefficient
// i: a byte of the block's literal plane string (see encode_block).  Entry = code word
// (bits 13:0) | length << 14 | (byte offset of the next state's 256 entries) << 18.
//
// Behind these, 256 entries that turn coefficient words into that literal string: entry a =
// eight planes of one coefficient, spread so that the plane at bit 7 - p of a lands on bit
// 4*p; coefficient i's entry is shifted up by i.
constexpr int kEncPlaneEntries = 5 * 256;
struct EncTable { uint32_t v[kEncPlaneEntries + 256]; };

constexpr EncTable build_enc_table() {
  EncTable t{};
  for (int n = 0; n <= 4; ++n)
    for (int x = 0; x < 256; ++x) {
      PlaneCode a = code_one_plane(n, x & 15);
      PlaneCode b = code_one_plane(a.next, x >> 4);
      t.v[n * 256 + x] = (a.code | b.code << a.len) | (uint32_t)(a.len + b.len) << 14 |
                         (uint32_t)(b.next * 256 * 4) << 18;
    }
  for (uint32_t a = 0; a < 256; ++a) {
    uint32_t e = 0;
    for (int p = 0; p < 8; ++p) e |= ((a >> (7 - p)) & 1u) << (4 * p);
    t.v[kEncPlaneEntries + a] = e;
  }
  return t;
}

// Encoder at rate 4, whole payload in one step.  Eight bits reach at most the first three
// non-empty planes in full (the first costs at least 3 bits, each later one at least 2) and
// of a fourth only the bit of coefficient 0, which comes first.  Index = those 13 bits:
// four planes of coefficient 0 (earliest plane highest), then three of coefficient 1, of
// coefficient 2, of coefficient 3.  Entry = the payload byte when the first of these
// planes is plane 31; with `lead` empty planes before it the payload is the entry shifted
// up by `lead` (an empty plane costs one zero bit; what no longer fits is cut, as the
// embedded code allows).  Planes below plane 0 enter the index as zeros and code as zeros,
// which is what unused payload bits are.
struct Enc4Table { uint8_t v[1 << 13]; };

constexpr Enc4Table build_enc4_table() {
  Enc4Table t{};
  for (int x = 0; x < (1 << 13); ++x) {
    const int c0 = (x >> 9) & 15, c1 = (x >> 6) & 7, c2 = (x >> 3) & 7, c3 = x & 7;
    uint32_t code = 0;
    int len = 0, n = 0;
    for (int k = 0; k < 4; ++k) {
      int p = (c0 >> (3 - k)) & 1;
      if (k < 3) p |= ((c1 >> (2 - k)) & 1) << 1 | ((c2 >> (2 - k)) & 1) << 2 | ((c3 >> (2 - k)) & 1) << 3;
      const PlaneCode a = code_one_plane(n, p);
      if (len < 32) code |= a.code << len;
      len += a.len;
      n = a.next;
    }
    t.v[x] = (uint8_t)(code & 0xFFu);
  }
  return t;
}

// Decoder tables for the planes read before three coefficients are significant (states
// 0, 1, 2; a fourth "idle" row of empty entries serves lanes that are past that point or out
// of budget, so that all lanes of a wavefront can step together).
//
// Entry (both tables): bits 1:0 of byte i = the bits of coefficient i in the planes read
// (the earlier plane in the higher bit) | planes read << 2 | stream bits used << 4 |
// (next state's row: 0, 1, 2 or 3 = idle) << 11.
//
// Look-ahead table: index = row*512 + next 9 stream bits, used when every lane that still
// reads has at least 9 bits of budget left, so that the budget cannot cut what an entry reads.
// An entry holds one plane, and a second one if that one also lies whole within the 9 bits
// and the first left the state below 3.
//
// Budget table: index = row*256 + (2^a - 1) + (next a stream bits), a = min(bits left, 7):
// one plane read with only a bits available, which resolves a code word cut by the budget (the
// one goes to the lowest index still possible); a = 0 reads nothing and leads to the idle row.
//
// Behind these, 256 entries for two planes at once when at least three coefficients are
// significant.  A plane is then four stream bits that are the plane's bits as they are
// (in state 3 the fourth is the group test of the one coefficient left, which is that
// coefficient's bit), whatever the state becomes.  Index = the next 8 stream bits; entry =
// for coefficient i, at bit 8*i, its bit of the first plane << 1 | its bit of the second.
constexpr int kDecLook = 9;
constexpr int kDecLookEntries = 4 << kDecLook;
constexpr int kDecBudgetEntries = 4 * 256;
constexpr int kDecPlaneEntries = kDecLookEntries + kDecBudgetEntries;
constexpr uint32_t kDecIdle = 3u << 11;   // state code of the idle row (the codes are the rows' byte offsets in the look-ahead table)
struct DecTable { uint32_t v[kDecPlaneEntries + 256]; };

constexpr uint32_t spread_planes(uint32_t first, uint32_t second, int planes) {
  uint32_t e = 0;
  for (int i = 0; i < 4; ++i) {
    const uint32_t b = planes == 2 ? (((first >> i) & 1u) << 1) | ((second >> i) & 1u) : (planes == 1 ? (first >> i) & 1u : 0u);
    e |= b << (8 * i);
  }
  return e;
}

constexpr DecTable build_dec_table() {
  DecTable t{};
  const uint32_t idle = 3u << 11;
  for (int n = 0; n < 3; ++n)
    for (int s = 0; s < (1 << kDecLook); ++s) {
      const PlaneBits a = read_one_plane(n, 16, (uint32_t)s);   // a plane is at most 7 bits long: always inside the 9
      uint32_t planes = 1, used = (uint32_t)a.used, bits = spread_planes(a.p, 0, 1);
      int next = a.next;
      if (a.next < 3) {
        const PlaneBits b = read_one_plane(a.next, 16, (uint32_t)s >> a.used);
        if (a.used + b.used <= kDecLook) {
          planes = 2;
          used += (uint32_t)b.used;
          bits = spread_planes(a.p, b.p, 2);
          next = b.next;
        }
      }
      t.v[(n << kDecLook) + s] = bits | planes << 2 | used << 4 | (next < 3 ? (uint32_t)next << 11 : idle);
    }
  for (int s = 0; s < (1 << kDecLook); ++s) t.v[(3 << kDecLook) + s] = idle;
  for (int n = 0; n < 3; ++n)
    for (int a = 0; a <= 7; ++a)
      for (int s = 0; s < (1 << a); ++s) {
        const PlaneBits r = read_one_plane(n, a, (uint32_t)s);
        const uint32_t e = a == 0 ? idle
                                  : spread_planes(r.p, 0, 1) | 1u << 2 | (uint32_t)r.used << 4 | (r.next < 3 ? (uint32_t)r.next << 11 : idle);
        t.v[kDecLookEntries + n * 256 + ((1 << a) - 1) + s] = e;
      }
  for (int s = 0; s < 256; ++s) t.v[kDecLookEntries + 3 * 256 + s] = idle;
  for (uint32_t b = 0; b < 256; ++b) {
    uint32_t e = 0;
    for (int i = 0; i < 4; ++i) e |= ((((b >> i) & 1u) << 1) | ((b >> (4 + i)) & 1u)) << (8 * i);
    t.v[kDecPlaneEntries + b] = e;
  }
  return t;
}

// Inverse of the lifting steps (wrap-around arithmetic, arithmetic shifts).
constexpr void inverse_lift(int32_t& a, int32_t& b, int32_t& c, int32_t& d) {
  auto add = [](int32_t p, int32_t q) { return (int32_t)((uint32_t)p + (uint32_t)q); };
  auto sub = [](int32_t p, int32_t q) { return (int32_t)((uint32_t)p - (uint32_t)q); };
  b = add(b, d); d = sub(d, b >> 2);
  d = sub(d, b >> 1); b = add(b, d);
  a = sub(a, c >> 1); c = add(c, a);
  c = sub(c, b >> 1); b = add(b, c);
  a = sub(a, d >> 1); d = add(d, a);
}

constexpr int32_t from_negabinary(uint32_t u) { return (int32_t)((u ^ 0xAAAAAAAAu) - 0xAAAAAAAAu); }

// Rate 4: the payload is one byte, so everything between the header and the final
// scaling is a function of 256 cases.  Entry = the four fixed-point values of the
// block divided by 2^22, as floats (4 floats per payload value): the values are multiples
// of 2^22 below 2^31 in magnitude, so the entries are small integers.  Eight payload bits reach at most planes
// 31..24 of the coefficient words.
struct Dec4Table { float v[256 * 4]; };

constexpr Dec4Table build_dec4_table() {
  Dec4Table t{};
  for (uint32_t payload = 0; payload < 256; ++payload) {
    uint32_t u[4] = {0, 0, 0, 0};
    int left = 8, n = 0;
    uint32_t s = payload;
    for (int k = 31; k >= 24 && left > 0; --k) {
      PlaneBits r = read_one_plane(n, left, s);
      for (int i = 0; i < 4; ++i) u[i] |= ((r.p >> i) & 1u) << k;
      s >>= r.used;
      left -= r.used;
      n = r.next;
    }
    int32_t a = from_negabinary(u[0]), b = from_negabinary(u[1]), c = from_negabinary(u[2]), d = from_negabinary(u[3]);
    inverse_lift(a, b, c, d);
    // multiples of 2^22 (the inverse lifting shifts multiples of 2^24 right by at most 2): kept
    // as that multiple, an integer below 2^9 in magnitude
    t.v[4 * payload + 0] = (float)(a >> 22);
    t.v[4 * payload + 1] = (float)(b >> 22);
    t.v[4 * payload + 2] = (float)(c >> 22);
    t.v[4 * payload + 3] = (float)(d >> 22);
  }
  return t;
}

// The same entries as IEEE half-precision bit patterns (integers below 2^9 are exact in a
// half's 11 significant bits), 8 bytes per payload value: the fused reduce reads these for
// every chunk after the first and feeds them to its multiply-add as they are (the GPU has a
// multiply-add that widens a half operand on the way in), which halves the LDS traffic of a
// look-up.
struct Dec4HalfTable { uint16_t v[256 * 4]; };

constexpr uint16_t small_int_as_half(int32_t x) {   // |x| < 2048
  if (x == 0) return 0;
  const uint32_t sign = x < 0 ? 0x8000u : 0u, m = (uint32_t)(x < 0 ? -x : x);
  int e = 0;
  while ((m >> (e + 1)) != 0) ++e;   // the exponent of the leading one, at most 10
  return (uint16_t)(sign | (uint32_t)(15 + e) << 10 | ((m << (10 - e)) & 0x3FFu));
}

constexpr Dec4HalfTable build_dec4_half_table() {
  const Dec4Table f = build_dec4_table();
  Dec4HalfTable t{};
  for (int i = 0; i < 256 * 4; ++i) t.v[i] = small_int_as_half((int32_t)f.v[i]);
  return t;
}

namespace selfcheck {
// every half-precision entry, widened by the format's definition, is the float entry
constexpr bool dec4_half_ok() {
  const Dec4Table f = build_dec4_table();
  const Dec4HalfTable h = build_dec4_half_table();
  for (int i = 0; i < 256 * 4; ++i) {
    const uint32_t b = h.v[i];
    int32_t v = 0;
    if (b & 0x7FFFu) {
      const int e = (int)((b >> 10) & 31u) - 15;          // 0 .. 10 for these entries
      if (e < 0 || e > 10) return false;
      const uint32_t m = 1024u + (b & 0x3FFu);            // 11 significant bits, worth m * 2^(e - 10)
      if ((m & ((1u << (10 - e)) - 1u)) != 0) return false;
      v = (int32_t)(m >> (10 - e));
    }
    if ((float)(b & 0x8000u ? -v : v) != f.v[i]) return false;
  }
  return true;
}
static_assert(dec4_half_ok(), "half-precision copy of the rate-4 block table");
}  // namespace selfcheck

// Pointers to the staged tables; a kernel sets only those its rate uses.
struct Tables {
  const uint32_t* enc;   // EncTable; at rate 4 the bytes of Enc4Table
  const uint32_t* dec;
  const float* dec4;
  const uint16_t* dec4_half;   // Dec4HalfTable (the fused reduce at rate 4)
};

template <int V>
struct IntConstant { static constexpr int value = V; };

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

// Four fp32 bit patterns -> biased block exponent E and the four negabinary
// coefficient words.  With m the largest magnitude as a bit pattern, E = (exponent
// field of m) + (m != 0): field + 1 for a normal maximum, 1 for a subnormal-only
// block, 0 for an all-zero block.  q_i = x_i * 2^(155 - E) truncated toward zero: the
// scaling is exact in fp32 (a result below 2^-126 may round, but truncates to 0 either
// way) and the float -> int conversion truncates.
ZC_DEV void forward_transform(const uint32_t (&x)[4], uint32_t& E, uint32_t (&u)[4]) {
  // largest magnitude as a bit pattern
#if defined(__HIP_DEVICE_COMPILE__)
  // For finite values the float maximum of the magnitudes is the same pattern as the integer
  // maximum of the patterns without their sign bits; the instructions take |x| as an operand
  // modifier (subnormals are kept: the kernels run with fp32 denormals on).
  float m3, mf;
  asm("v_max3_f32 %0, |%1|, |%2|, |%3|" : "=v"(m3) : "v"(bits_to_float(x[0])), "v"(bits_to_float(x[1])), "v"(bits_to_float(x[2])));
  asm("v_max_f32_e64 %0, |%1|, |%2|" : "=v"(mf) : "v"(m3), "v"(bits_to_float(x[3])));
  const uint32_t m = __builtin_bit_cast(uint32_t, mf);
#else
  const uint32_t m = umax(umax(x[0] & 0x7FFFFFFFu, x[1] & 0x7FFFFFFFu), umax(x[2] & 0x7FFFFFFFu, x[3] & 0x7FFFFFFFu));
#endif
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

// Whole block: exponent byte + embedded code of the coefficients, cut at the budget.
// `any_lane_active(pred)` tells whether any lane of the wavefront still has pred set
// (loop control only); any_lane_active.lanes(pred) is the set of those lanes and
// any_lane_active.some(set) whether a set is non-empty, for votes on several comparisons
// at once (each comparison's own result is such a set, and sets combine for free).
//
// Rates above 4 encode in two phases, around the block's literal plane string: the planes
// from the first non-empty one down, four bits each in coefficient order, which is what
// the stream holds from the moment three coefficients are significant (a plane is then
// its four bits as they are).  (1) While any lane with bits left is in a state below 3,
// all lanes code two planes per step through the table, indexed by the next byte of the
// literal string.  (2) What is left of the budget is filled from the literal string itself:
// one funnel shift puts the bits of phase 1 and the literal bits behind them in place and
// cuts at the block's end.  (Planes past plane 0 enter the string as zeros and code as
// zeros, which is what unused bits are.)
template <int RATE, class AnyActive>
ZC_DEV void encode_block(const uint32_t (&x)[4], const Tables& tab, uint32_t (&W)[Traits<RATE>::kWords],
                         AnyActive any_lane_active) {
  constexpr int NW = Traits<RATE>::kWords;
  constexpr int kPayload = Traits<RATE>::kPayloadBits;
  // every plane costs at least one bit, so at most this many planes are ever coded
  constexpr int kMaxPlanes = kPayload < 32 ? kPayload : 32;
  constexpr int kLitWords = (kMaxPlanes + 7) / 8;
  uint32_t E, u[4];
  forward_transform(x, E, u);
  // leading empty planes: one zero bit each
  // (at rate 4 the count only serves as a shift of the words and of the table's entry, which are
  // zero when all words are)
  const uint32_t lead = RATE == 4 ? count_leading_zeros_nonzero(u[0] | u[1] | u[2] | u[3])
                                  : count_leading_zeros(u[0] | u[1] | u[2] | u[3]);
  const int32_t avail = kPayload - (int32_t)lead;
  uint32_t left = avail > 0 ? (uint32_t)avail : 0u;
#pragma unroll
  for (int i = 0; i < 4; ++i) u[i] <<= (lead & 31u);  // top plane to bit 31 (all words are zero if lead = 32)
  if constexpr (RATE == 4) {
    uint32_t idx = u[0] >> 28;
    idx = alignbit(idx, u[1], 29);  // (idx << 3) | top three bits of the next word
    idx = alignbit(idx, u[2], 29);
    idx = alignbit(idx, u[3], 29);
    const uint32_t payload = ((uint32_t) reinterpret_cast<const uint8_t*>(tab.enc)[idx] << (lead & 31u)) & 0xFFu;
    W[0] = E | payload << 8;
    (void)left;
    (void)any_lane_active;
    return;
  } else {
    // the literal plane string: byte t of it = planes 2t and 2t+1.  Its words are made when they
    // are first needed: word 0 now, a later word when phase 1 reaches it or when some lane's
    // remaining budget reaches into it.
    const uint32_t* spread = tab.enc + kEncPlaneEntries;
    uint32_t lit[kLitWords];
    auto make_word = [&](int j) {
      const int sh = 24 - 8 * j;
      lit[j] = spread[(u[0] >> sh) & 0xFFu] | spread[(u[1] >> sh) & 0xFFu] << 1 | spread[(u[2] >> sh) & 0xFFu] << 2 |
               spread[(u[3] >> sh) & 0xFFu] << 3;
    };
    make_word(0);
#pragma unroll
    for (int j = 1; j < kLitWords; ++j) lit[j] = 0u;
    // phase 1: code words enter at the top of the window P, older bits move down
    uint32_t P[NW];
#pragma unroll
    for (int j = 0; j < NW; ++j) P[j] = 0;
    uint32_t state = 0;   // byte offset of the current state's table rows
    uint32_t steps = 0;   // the same in every lane
    int made = 1;         // words of the literal string made so far (the same in every lane)
    bool open = true;
#pragma unroll
    for (int w = 0; w < kLitWords; ++w) {
      if (open) {
        if (w > 0 && any_lane_active.some(any_lane_active.lanes(left > 0) & any_lane_active.lanes(state < 3u * 256u * 4u))) {
          make_word(w);
          made = w + 1;
        }
        uint32_t z = lit[w], togo = 4u;   // steps this word still has bytes for
#pragma unroll 1
        while (togo != 0u && any_lane_active.some(any_lane_active.lanes(left > 0) & any_lane_active.lanes(state < 3u * 256u * 4u))) {
          --togo;
          ++steps;
          uint32_t byte = z & 0xFFu;
          materialise(byte);   // (so that the address is this byte shifted and added to the row's offset in one instruction)
          const uint32_t e = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(tab.enc) + state + (byte << 2));
          z >>= 8;
          const uint32_t len = umin((e >> 14) & 15u, left);
          shift_in<NW>(P, e, len);  // only the low `len` bits of e enter the window
          left -= len;
          state = e >> 18;
        }
        open = togo == 0u;
      }
    }
    // word j of the string is needed below iff some lane's budget reaches past bit 32*j of it
    {
      bool further = true;
#pragma unroll
      for (int j = 1; j < kLitWords; ++j) {
        if (further) {
          further = any_lane_active(left + 8u * steps > 32u * (uint32_t)j);
          if (further && j >= made) make_word(j);
        }
      }
    }
    // phase 2: X = the window of phase 1 with the literal string from byte `steps` on above it
    uint32_t X[2 * NW];
#pragma unroll
    for (int j = 0; j < NW; ++j) X[j] = P[j];
    const uint32_t byte_shift = 8u * (steps & 3u);
    auto literal_from = [&](auto first_word) {
      constexpr int w0 = decltype(first_word)::value;
#pragma unroll
      for (int j = 0; j < NW; ++j) {
        const uint32_t lo = w0 + j < kLitWords ? lit[w0 + j < kLitWords ? w0 + j : 0] : 0u;
        const uint32_t hi = w0 + j + 1 < kLitWords ? lit[w0 + j + 1 < kLitWords ? w0 + j + 1 : 0] : 0u;
        X[NW + j] = alignbit(hi, lo, byte_shift);
      }
    };
    switch (steps >> 2) {
      case 0: literal_from(IntConstant<0>()); break;
      case 1: literal_from(IntConstant<1>()); break;
      case 2: literal_from(IntConstant<2>()); break;
      case 3: literal_from(IntConstant<3>()); break;
      default: literal_from(IntConstant<4>()); break;
    }
    // the coded bits of phase 1 sit at the top of P and the first of them belongs at bit
    // 8 + lead: everything moves down by the unused budget (and by the window's excess
    // over the block), which brings exactly `left` literal bits into the block
    const uint32_t down = (uint32_t)(32 * NW - Traits<RATE>::kBlockBits) + left;
    const uint32_t r = down & 31u, k = down >> 5;
    uint32_t F[2 * NW - 1];
#pragma unroll
    for (int j = 0; j < 2 * NW - 1; ++j) F[j] = alignbit(X[j + 1], X[j], r);
#pragma unroll
    for (int o = 0; o < NW; ++o) {
      uint32_t v = F[o];
#pragma unroll
      for (int d = 1; d < NW; ++d) v = (k == (uint32_t)d) ? F[o + d] : v;
      W[o] = v;
    }
    if constexpr (Traits<RATE>::kBlockBits % 32 != 0) W[NW - 1] &= (1u << (Traits<RATE>::kBlockBits % 32)) - 1u;
    W[0] |= E;
  }
}

// ---- inverse path ------------------------------------------------------------------

// (u xor 0xAAAAAAAA) - 0xAAAAAAAA; on the device one xor-add instruction (its two constants
// cannot both be immediates, so one sits in a scalar and one in a vector register).
ZC_DEV int32_t negabinary_to_int(uint32_t u) {
#if defined(__HIP_DEVICE_COMPILE__)
  uint32_t r;
  asm("v_xad_u32 %0, %1, %2, %3" : "=v"(r) : "v"(u), "s"(0xAAAAAAAAu), "v"(0x55555556u));
  return (int32_t)r;
#else
  return from_negabinary(u);
#endif
}

ZC_DEV void inverse_transform(const uint32_t (&u)[4], uint32_t E, float (&out)[4]) {
  int32_t a = negabinary_to_int(u[0]), b = negabinary_to_int(u[1]), c = negabinary_to_int(u[2]), d = negabinary_to_int(u[3]);
  inverse_lift(a, b, c, d);
  const int ex = (int)E - 127 - kFractionBits;
  // int -> fp32 rounds to nearest even; the scaling is exact and rounds once more only
  // for subnormal results.  A zero block arrives here with all words zero: +0.
  out[0] = __builtin_ldexpf((float)a, ex);
  out[1] = __builtin_ldexpf((float)b, ex);
  out[2] = __builtin_ldexpf((float)c, ex);
  out[3] = __builtin_ldexpf((float)d, ex);
}

// W holds the block (bits beyond 4*RATE zero).
//
// Rates above 4 decode in two phases.  (1) While any lane of the wavefront is in a state
// below 3 with bits left, all lanes step together through the tables: one or two planes per
// step from the look-ahead table, or, when some reading lane is within 9 bits of its budget,
// one plane from the budget table; lanes past that point take empty entries.  (2) From state 3
// on a plane is four stream bits that are the plane's bits as they are (in state 3 the fourth
// is the group test of the one coefficient left, which is that coefficient's bit), and bits
// past the budget are zeros in the window and decode as the zeros that unseen bits are; so
// the rest of the window is taken as it stands, eight planes per 32 bits through the pair
// table, with no loop, no budget and no state, and joined to the planes of phase 1.
template <int RATE, class AnyActive>
ZC_DEV void decode_block(uint32_t (&W)[Traits<RATE>::kWords], const Tables& tab, float (&out)[4],
                         AnyActive any_lane_active) {
  constexpr int NW = Traits<RATE>::kWords;
  constexpr int kPayload = Traits<RATE>::kPayloadBits;
  const uint32_t E = W[0] & 0xFFu;
  if constexpr (RATE == 4) {
    // one lookup for the whole payload byte (entry 0 is the zero block, which ignores
    // its payload), then only the scaling by 2^(E - 155) is left
    const float* q = tab.dec4 + 4u * (E ? W[0] >> 8 : 0u);
    const int ex = (int)E - 127 - kFractionBits + 22;
#pragma unroll
    for (int i = 0; i < 4; ++i) out[i] = __builtin_ldexpf(q[i], ex);
  } else {
    // literal words of phase 2: at least one bit is gone after phase 1, and at most 31 planes remain
    constexpr int kLiteral = (kPayload - 1 + 31) / 32 < 4 ? (kPayload - 1 + 31) / 32 : 4;
    // leading empty planes = zero bits at the start of the payload
    uint32_t lead = 0;
    {
      bool found = false;
#pragma unroll
      for (int j = 0; j < NW; ++j) {
        const uint32_t w = j == 0 ? (W[0] & 0xFFFFFF00u) : W[j];
        const uint32_t z = count_trailing_zeros(w);
        lead = found ? lead : lead + z;
        found = found || (w != 0);
      }
      lead -= 8u;  // the header byte
    }
    lead = umin(lead, (uint32_t)kPayload);
    uint32_t left = (uint32_t)kPayload - lead;
    // keep the next stream bit at bit 2 of the window: bits 10..2 index the look-ahead table directly.
    // Two shifts of less than 32 each (a block with 32 and more leading empty planes has its
    // window cleared below, so there only the low five bits of the count need to act).
    shift_out<NW>(W, 6u);
    shift_out<NW>(W, lead & 31u);
    uint32_t state = 0;
    // a zero block ignores its payload; after 32 empty planes nothing is left to decode
    if (E == 0u || (kPayload > 32 && lead >= 32u)) {
      left = 0u;
      lead = 0u;
      state = kDecIdle;
#pragma unroll
      for (int j = 0; j < NW; ++j) W[j] = 0u;
    }
    // phase 1.  A[i] collects the planes of coefficient i, the latest in bit 0; m counts them
    // (per lane: a step reads one or two planes, or none in a lane that is idle).
    uint32_t A[4] = {0u, 0u, 0u, 0u}, m = 0;
    // one group of up to four steps: byte i of acc = the group's planes of coefficient i (at most eight)
    auto group = [&](uint32_t& acc, uint32_t& mg) {
      uint32_t s = 0;
#pragma unroll 1
      for (; s < 4u; ++s) {
        const auto reading = any_lane_active.lanes(state < kDecIdle);
        if (!any_lane_active.some(reading)) break;
        // byte offset of the entry (the state code is the row's byte offset in the look-ahead
        // table, eight times the row's in the budget table; the next stream bit is bit 2 of W[0])
        uint32_t at;
        if (any_lane_active.some(reading & any_lane_active.lanes(left < (uint32_t)kDecLook))) {
          const uint32_t mask4 = (4u << umin(left, 7u)) - 4u;   // the next min(left, 7) stream bits, in place
          at = 4u * kDecLookEntries + (state >> 1) + mask4 + (W[0] & mask4);
        } else {
          at = state | (W[0] & (((1u << kDecLook) - 1u) << 2));
        }
        const uint32_t e = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(tab.dec) + at);
        const uint32_t planes = (e >> 2) & 3u, used = (e >> 4) & 15u;
        acc = (acc << planes) | (e & 0x03030303u);
        mg += planes;
        shift_out<NW>(W, used);
        left -= used;
        state = e & kDecIdle;
      }
      return s == 4u;
    };
    {
      uint32_t acc = 0;
      bool open = group(acc, m);
#pragma unroll
      for (int i = 0; i < 4; ++i) A[i] = (acc >> (8 * i)) & 0xFFu;
      // more groups only for blocks that stay below three significant coefficients for long; no
      // more than 32 planes are kept (a block has no more, whatever the stream goes on to say)
#pragma unroll 1
      for (int g = 1; g < 8 && open; ++g) {
        uint32_t mg = 0;
        acc = 0;
        open = group(acc, mg);
        const uint32_t take = umin(mg, 32u - m);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const uint32_t planes = ((acc >> (8 * i)) & 0xFFu) >> (mg - take);
          A[i] = take >= 32u ? planes : (A[i] << take) | planes;
        }
        m += take;
      }
    }
    // phase 2.  G[j]: byte i = the next eight literal planes of coefficient i, the first in bit 7
    uint32_t u[4];
    {
      const uint32_t* pair = tab.dec + kDecPlaneEntries;
      uint32_t G[kLiteral];
#pragma unroll
      for (int j = 0; j < kLiteral; ++j) {
        uint32_t bits = W[j] >> 2;
        if (j + 1 < NW) bits = alignbit(W[j + 1], W[j], 2);
        G[j] = pair[bits & 0xFFu] << 6 | pair[(bits >> 8) & 0xFFu] << 4 | pair[(bits >> 16) & 0xFFu] << 2 | pair[bits >> 24];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        // the literal planes of coefficient i from bit 31 down
        uint32_t B;
        if constexpr (kLiteral == 1) {
          B = permute_bytes(0u, G[0], 0x000c0c0cu | (uint32_t)i << 24);
        } else {
          B = permute_bytes(G[0], G[1], 0x00000c0cu | (uint32_t)(4 + i) << 24 | (uint32_t)i << 16);
          if constexpr (kLiteral == 3) B = permute_bytes(B, G[2], 0x0706000cu | (uint32_t)i << 8);
          if constexpr (kLiteral == 4) B |= permute_bytes(G[2], G[3], 0x0c0c0000u | (uint32_t)(4 + i) << 8 | (uint32_t)i);
        }
        u[i] = B;
      }
      // the m planes of phase 1 above the literal ones, and all of it down by the empty planes:
      // one funnel shift while m + lead stays below 32
      const uint32_t down = m + lead;
      if (any_lane_active(down > 31u)) {
#pragma unroll
        for (int i = 0; i < 4; ++i) u[i] = (m >= 32u ? A[i] : alignbit(A[i], u[i], m)) >> lead;
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) u[i] = alignbit(A[i], u[i], down);
      }
    }
    inverse_transform(u, E, out);
  }
}

// Rate 4 in the fused reduce: sum = (FIRST) or sum += (otherwise) the decoded block, with one
// rounding per value as a decode followed by an add would give.
//
// Plain form, for exponent bytes 1..249 and for zero blocks whose payload is zero: the table's
// entries are integers below 2^9 and 2^(E - 133) is a representable (possibly subnormal) power
// of two, so their product is exact and the fused multiply-add rounds the same sum once; entry 0
// is four zeros, so a zero block with a zero payload needs no test of its exponent byte.
template <bool FIRST>
ZC_DEV void accumulate_plain4(uint32_t W0, const Tables& tab, float (&sum)[4]) {
  const int ex = (int)(W0 & 0xFFu) - 127 - kFractionBits + 22;
  if constexpr (FIRST) {
    const float* q = reinterpret_cast<const float*>(reinterpret_cast<const char*>(tab.dec4) + (((W0 >> 8) & 0xFFu) << 4));
#pragma unroll
    for (int i = 0; i < 4; ++i) sum[i] = __builtin_ldexpf(q[i], ex);
  } else {
    const float scale = __builtin_ldexpf(1.0f, ex);
    const char* entry = reinterpret_cast<const char*>(tab.dec4_half) + (((W0 >> 8) & 0xFFu) << 3);
#ifdef __HIP_DEVICE_COMPILE__
    // eight bytes, four halves; widening a half is exact, so each line is the same fused
    // multiply-add as on the float entry (one instruction: the half is widened inside it)
    typedef _Float16 HalfPair __attribute__((ext_vector_type(2)));
    typedef uint32_t WordPair __attribute__((ext_vector_type(2)));
    const WordPair raw = *reinterpret_cast<const WordPair*>(entry);
    // (the two words go through scalars of their own: a bit cast applied to a vector's
    // component directly took the first component both times with this compiler)
    const uint32_t first = raw.x, second = raw.y;
    const HalfPair lo = __builtin_bit_cast(HalfPair, first), hi = __builtin_bit_cast(HalfPair, second);
    sum[0] = __builtin_fmaf((float)lo.x, scale, sum[0]);
    sum[1] = __builtin_fmaf((float)lo.y, scale, sum[1]);
    sum[2] = __builtin_fmaf((float)hi.x, scale, sum[2]);
    sum[3] = __builtin_fmaf((float)hi.y, scale, sum[3]);
#else
    const uint16_t* h = reinterpret_cast<const uint16_t*>(entry);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      // a normal half or zero: (1 + fraction / 1024) * 2^(exponent - 15)
      const float q = h[i] & 0x7FFFu ? __builtin_ldexpf((float)(1024 + (h[i] & 0x3FFu)), (int)((h[i] >> 10) & 31u) - 25) : 0.0f;
      sum[i] = __builtin_fmaf(h[i] & 0x8000u ? -q : q, scale, sum[i]);
    }
#endif
  }
}

// Careful form, for any block: a zero exponent byte ignores the payload, and the decoded value
// is rounded (possibly to infinity: from E = 252 on the product overflows) before it is added.
// Only arbitrary bytes or values of 2^127 and more produce blocks that need it.
template <bool FIRST>
ZC_DEV void accumulate_careful4(uint32_t W0, const Tables& tab, float (&sum)[4]) {
  const uint32_t E = W0 & 0xFFu;
  const float* q = tab.dec4 + 4u * (E ? (W0 >> 8) & 0xFFu : 0u);
  const int ex = (int)E - 127 - kFractionBits + 22;
#pragma unroll
  for (int i = 0; i < 4; ++i) sum[i] = FIRST ? __builtin_ldexpf(q[i], ex) : sum[i] + __builtin_ldexpf(q[i], ex);
}

// Whether a block (W0 = its two bytes, zero-extended) is outside what the plain form covers:
// exponent byte 250 and more, or exponent byte 0 over a nonzero payload.  W0 - 1 has 255 in
// its low byte in the second case and E - 1 otherwise; the all-zero block wraps to a word with
// the top bit set, which the signed compare leaves out.
ZC_DEV bool unusual4(uint32_t W0) { return (int32_t)((W0 - 1u) & 0x800000FFu) >= 249; }

// ---- tile order of the wide rate-4 decompress kernel ---------------------------------
// That kernel is bound by its non-temporal stores of the fp32 output, and how the
// workgroups' tiles are spread over the buffer matters a little for those (measured with
// plain store kernels: 4 to 9 % faster when each XCD writes whole 1 MiB regions than under a
// plain grid stride; in the kernel itself 2 %; for reads, and for the kernels at the other
// rates, the order makes no difference).  Workgroup b runs on XCD b mod 8, so the
// grid-stride index v = b + k * grid (grid a multiple of 8) is turned into a tile number
// such that the tiles with v mod 8 = x are, in order, the tiles of regions x, x + 8, ... of
// 2^lg tiles each.  Indices from `bulk` on (what does not fill eight regions) stay as they
// are; the map is one-to-one on [0, bulk).
ZC_DEV constexpr size_t region_bulk(size_t tiles, int lg) { return (tiles >> (lg + 3)) << (lg + 3); }

ZC_DEV size_t region_order(size_t v, size_t bulk, int lg) {
  if (v >= bulk) return v;
  const size_t q = v >> 3, x = v & 7;
  return ((((q >> lg) << 3) + x) << lg) + (q & (((size_t)1 << lg) - 1));
}

}  // namespace zc
#endif  // ZC_CODEC_H
