// zc2d_codec.h -- per-block codec for 4 x 4 blocks ("ZC-2D"), as run by one GPU lane.
//
// Same codec family as zc_codec.h (the paper's lossy fixed-rate compressor of the ZFP
// kind, Sec. II-A, Sec. III-B) for matrix-shaped messages: shared exponent of the 16
// values, truncating conversion to 27 fraction bits, the reversible lifting transform
// along rows and then along columns, coefficients in order of total sequency,
// negabinary digits, and the embedded bit-plane code with 16 coefficients, cut at
// 16*RATE-8 bits behind a one-byte exponent header.
//
// How the bit-plane code is computed here:
//   * the words are aligned so that the first non-empty plane is bit 31, and their upper
//     halves are bit-transposed (a 16 x 16 transpose on eight registers that hold two
//     16-bit rows each), so that each of the first 16 planes is one 16-bit pattern in a
//     register; the lower halves are transposed only if some lane of the wavefront gets
//     that far within its budget, which low rates rarely do;
//   * the plane loop is unrolled, uniform over the wavefront, and ends when no lane has
//     budget left;
//   * encoder: the group tests of a plane are computed without a loop.  In the stream
//     the newly significant coefficient of index p (counted from the first coefficient
//     not yet significant) and rank j (1-based) ends its token at bit p + j, and every
//     token starts one bit after the previous one ended, so the code is the pattern
//     with each one moved up by its rank (two look-ups in a 256-entry table) plus that
//     word shifted by one;
//   * decoder: a table indexed by the next 9 stream bits and by how far the last
//     coefficient is (whose token has no closing one) decodes all the tokens that lie
//     whole within those bits; it is used when its result stays inside the budget,
//     otherwise one token is decoded by count-trailing-zeros with the limits applied.
//     A budget cut inside a run places the decoded one after the zeros read so far, which
//     is the lowest index still possible.  A lane's progress through a plane is one state
//     word that table entries are added to; lanes whose plane is closed read an all-zero
//     row, so that a step needs no per-lane case distinction;
//   * after the planes, the usual case (at most 16 planes read, starting within the top
//     16) turns each coefficient's 16-bit pattern into its word with one shift.
#ifndef ZC2D_CODEC_H
#define ZC2D_CODEC_H

#include "zc_codec.h"

namespace zc2d {

using zc::alignbit;
using zc::umin;
using zc::umax;
using zc::count_leading_zeros;
using zc::count_trailing_zeros;

constexpr int kFractionBits = 27;

template <int RATE>
struct Traits {
  static_assert(RATE == 2 || RATE == 4 || RATE == 8 || RATE == 16, "rate");
  static constexpr int kBlockBits = 16 * RATE;
  static constexpr int kBlockBytes = 2 * RATE;
  static constexpr int kPayloadBits = 16 * RATE - 8;
  static constexpr int kWords = RATE / 2;
};

// Position of coefficient c in the 4 x 4 array (4*i + j, i = row frequency, j = column
// frequency): ascending i + j, ties by ascending i.
struct Order { int v[16]; };
constexpr Order build_order() {
  Order o{};
  int c = 0;
  for (int s = 0; s <= 6; ++s)
    for (int i = 0; i < 4; ++i) {
      int j = s - i;
      if (j >= 0 && j < 4) o.v[c++] = 4 * i + j;
    }
  return o;
}
constexpr Order kOrder = build_order();

// ---- 16 x 16 bit transpose on eight words ----------------------------------------------
// Row r of a 16 x 16 bit matrix sits in half r >> 3 of word r & 7 (half 0 = bits 0..15).
// The transpose leaves the matrix in the same arrangement, so it is its own inverse.
// WHOLE: all eight results are needed (the decoder), so the byte swap is one permute per word;
// otherwise plain bit operations throughout, which lets the compiler compute only what the
// planes actually coded ask for (the encoder, which at low rates codes few of the 16).
template <bool WHOLE>
ZC_DEV constexpr void transpose_halves(uint32_t (&a)[8]) {
  // swap the 8 x 8 quadrants: bits 8..15 of row r with bits 0..7 of row r + 8 (the two middle
  // bytes of each word change places)
#pragma unroll
  for (int w = 0; w < 8; ++w) {
    if (!WHOLE || __builtin_is_constant_evaluated())
      a[w] = (a[w] & 0xFF0000FFu) | ((a[w] & 0x0000FF00u) << 8) | ((a[w] >> 8) & 0x0000FF00u);
    else
      a[w] = zc::permute_bytes(a[w], a[w], 0x03010200u);
  }
  // then 4 x 4, 2 x 2 and 1 x 1 blocks between words j apart; each mask's complement is the
  // mask shifted up by j, so a result is one shift and one bit-field insert
  constexpr uint32_t mask[3] = {0x0F0F0F0Fu, 0x33333333u, 0x55555555u};
  int m = 0;
#pragma unroll
  for (int j = 4; j >= 1; j >>= 1, ++m)
#pragma unroll
    for (int w = 0; w < 8; ++w)
      if ((w & j) == 0) {
        const uint32_t lo = a[w], hi = a[w + j];
        a[w] = (lo & mask[m]) | ((hi << j) & ~mask[m]);
        a[w + j] = ((lo >> j) & mask[m]) | (hi & ~mask[m]);
      }
}

// ---- tables --------------------------------------------------------------------------
// Encoder: v[c] has, for each one of c at position p with 1-based rank j, bit p + j set.
struct ExpandTable { uint32_t v[256]; };
constexpr ExpandTable build_expand_table() {
  ExpandTable t{};
  for (int c = 0; c < 256; ++c) {
    uint32_t e = 0;
    int rank = 0;
    for (int p = 0; p < 8; ++p)
      if ((c >> p) & 1) { ++rank; e |= 1u << (p + rank); }
    t.v[c] = e;
  }
  return t;
}

// Decoder: entry for the next kLookahead stream bits at the start of a group test, by how far
// the last coefficient is.  The decoder keeps, per plane, a state s = (index of the first
// coefficient not yet known to be significant) | (plane closed) << 5 and looks up row
// clamp(s, 6, 16) - 6: row 0 serves the indices up to 6, from where the last coefficient
// cannot be reached within the look-ahead; rows 1..9 are the indices 7..15 (8..0 coefficients
// between the current one and the last); row 10, all zeros, is what a lane reads whose plane is
// closed (a closing zero was read, or the last coefficient dealt with), so that it can step
// along with the others and nothing happens.
// An entry holds all the tokens that lie whole within the look-ahead: group bit, zeros,
// closing one; a run that reaches the last coefficient needs no closing one, and the plane is
// closed after it; a group bit 0 closes the plane.
// Bits 0..9: the ones, as positions past the current coefficient; bits 10..14: how many
// coefficients were passed; bit 15: the plane is closed (bits 10..15 are added to s);
// bits 20..23: how many stream bits were used; bit 31: no token ends within the look-ahead
// (so that entry >> 20 exceeds any budget, and the decoder reads one token on its own).
constexpr int kLookahead = 9;
constexpr int kTokenRows = 11;
constexpr uint32_t kTokenFirstRowState = 6, kTokenIdleState = 16;
struct TokenTable { uint32_t v[kTokenRows << kLookahead]; };
constexpr TokenTable build_token_table() {
  TokenTable t{};
  for (uint32_t row = 0; row + 1 < (uint32_t)kTokenRows; ++row) {
    // coefficients between the current one and the last; row 0 stands for nine and more
    const uint32_t room = row == 0 ? 15u : 9u - row;
    for (uint32_t s = 0; s < (1u << kLookahead); ++s) {
      uint32_t ones = 0, passed = 0, used = 0, done = 0;
      for (;;) {
        if (passed > room) { done = 1; break; }             // the last coefficient has been dealt with
        if (used >= (uint32_t)kLookahead) break;
        if (((s >> used) & 1u) == 0u) { done = 1; ++used; break; }
        uint32_t z = 0;
        bool in_sight = true;
        while (passed + z < room) {
          if (used + 1 + z >= (uint32_t)kLookahead) { in_sight = false; break; }
          if ((s >> (used + 1 + z)) & 1u) break;
          ++z;
        }
        if (!in_sight) break;
        ones |= 1u << (passed + z);
        used += 1 + z + (passed + z == room ? 0 : 1);       // no closing one at the last coefficient
        passed += z + 1;
      }
      t.v[(row << kLookahead) + s] = ones | passed << 10 | done << 15 | used << 20 | (used == 0u ? 1u << 31 : 0u);
    }
  }
  return t;
}

namespace selfcheck {
template <bool WHOLE>
constexpr bool transpose_ok() {
  uint32_t a[8] = {}, ref[8] = {};
  uint32_t s = 0x9E3779B9u;
  for (int w = 0; w < 8; ++w) { s = s * 1664525u + 1013904223u; a[w] = s; }
  for (int r = 0; r < 16; ++r)
    for (int b = 0; b < 16; ++b)
      ref[b & 7] |= ((a[r & 7] >> (16 * (r >> 3) + b)) & 1u) << (16 * (b >> 3) + r);
  transpose_halves<WHOLE>(a);
  for (int w = 0; w < 8; ++w)
    if (a[w] != ref[w]) return false;
  return true;
}
static_assert(transpose_ok<true>() && transpose_ok<false>(), "16 x 16 bit transpose");
}  // namespace selfcheck

// ---- forward ---------------------------------------------------------------------------

ZC_DEV void lift_forward(int32_t& a, int32_t& b, int32_t& c, int32_t& d) {
  d -= a; a += d >> 1;
  b -= c; c += b >> 1;
  c -= a; a += c >> 1;
  b -= d; d += b >> 1;
  d += b >> 2; b -= d;
}

// x: the block row-major as fp32 bit patterns.  Returns E and the negabinary words in
// coefficient order.
ZC_DEV void forward_transform(const uint32_t (&x)[16], uint32_t& E, uint32_t (&u)[16]) {
  // largest magnitude as a bit pattern (on the device a float maximum with |x| operands, as in
  // the 1-D codec: the same pattern for finite values, a third of the instructions)
#if defined(__HIP_DEVICE_COMPILE__)
  float mf = 0.0f;
#pragma unroll
  for (int i = 0; i < 16; i += 2)
    asm("v_max3_f32 %0, |%1|, |%2|, |%3|" : "=v"(mf) : "v"(mf), "v"(zc::bits_to_float(x[i])), "v"(zc::bits_to_float(x[i + 1])));
  const uint32_t m = __builtin_bit_cast(uint32_t, mf);
#else
  uint32_t m = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i) m = umax(m, x[i] & 0x7FFFFFFFu);
#endif
  E = (m >> 23) + (m != 0u ? 1u : 0u);
  const int scale = 127 + kFractionBits - (int)E;
  int32_t q[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) q[i] = (int32_t)__builtin_ldexpf(zc::bits_to_float(x[i]), scale);
#pragma unroll
  for (int r = 0; r < 4; ++r) lift_forward(q[4 * r], q[4 * r + 1], q[4 * r + 2], q[4 * r + 3]);
#pragma unroll
  for (int c = 0; c < 4; ++c) lift_forward(q[c], q[4 + c], q[8 + c], q[12 + c]);
#pragma unroll
  for (int c = 0; c < 16; ++c) u[c] = ((uint32_t)q[kOrder.v[c]] + 0xAAAAAAAAu) ^ 0xAAAAAAAAu;
}

// One plane of the embedded code.  pat: the plane's bit of each coefficient; n: how many
// leading coefficients are significant; left: budget.  Appends to the window W.
template <int NW>
ZC_DEV void encode_plane(uint32_t pat, const uint32_t* expand, uint32_t (&W)[NW], uint32_t& n, uint32_t& left) {
  // coefficients already significant: their bits as they are
  const uint32_t vlen = umin(n, left);
  zc::shift_in<NW>(W, pat, vlen);
  left -= vlen;
  // the rest: ends of the tokens, then their starts one bit after the previous end
  const uint32_t rest = pat >> n;
  const uint32_t lo = expand[rest & 0xFFu], hi = expand[rest >> 8];
  const uint32_t ends = lo | hi << (8u + (uint32_t)__builtin_popcount(rest & 0xFFu));
  const uint32_t last = 31u - count_leading_zeros(ends);      // wraps to -1 if there is none
  const uint32_t starts = ((ends << 1) & ((1u << (last & 31u)) - 1u)) | umin(ends, 1u);
  uint32_t len = last + 2u;              // up to the last end, and the closing group bit 0
  if (pat >> 15) len -= 2u;              // the last coefficient needs neither its end nor a closing bit
  if (n == 16u) len = 0u;                // (when n is 16 the bit tested above was not a new one)
  const uint32_t glen = umin(len, left);
  zc::shift_in<NW>(W, ends | starts, glen);
  left -= glen;
  n = umax(n, 32u - count_leading_zeros(pat));
}

template <int RATE, class AnyActive>
ZC_DEV void encode_block(const uint32_t (&x)[16], const uint32_t* expand, uint32_t (&W)[Traits<RATE>::kWords],
                         AnyActive any_lane_active) {
  constexpr int NW = Traits<RATE>::kWords;
  constexpr int kMaxPlanes = Traits<RATE>::kPayloadBits < 32 ? Traits<RATE>::kPayloadBits : 32;
  uint32_t E, u[16];
  forward_transform(x, E, u);
  uint32_t any = 0;
#pragma unroll
  for (int c = 0; c < 16; ++c) any |= u[c];
  const uint32_t lead = count_leading_zeros(any);   // empty planes: one zero bit each
  const int32_t avail = Traits<RATE>::kPayloadBits - (int32_t)lead;
  uint32_t left = avail > 0 ? (uint32_t)avail : 0u;
#pragma unroll
  for (int c = 0; c < 16; ++c) u[c] <<= (lead & 31u);   // first non-empty plane to bit 31
#pragma unroll
  for (int j = 0; j < NW; ++j) W[j] = 0;
  uint32_t n = 0;
  uint32_t h[8];
#pragma unroll
  for (int w = 0; w < 8; ++w) h[w] = (u[w] >> 16) | (u[w + 8] & 0xFFFF0000u);
  transpose_halves<false>(h);
#pragma unroll
  for (int t = 0; t < 16; ++t) {
    if (t >= kMaxPlanes || !any_lane_active(left > 0)) break;
    const int b = 15 - t;
    encode_plane<NW>((b >> 3) ? h[b & 7] >> 16 : h[b & 7] & 0xFFFFu, expand, W, n, left);
  }
  if (kMaxPlanes > 16 && any_lane_active(left > 0)) {
#pragma unroll
    for (int w = 0; w < 8; ++w) h[w] = (u[w] & 0xFFFFu) | (u[w + 8] << 16);
    transpose_halves<false>(h);
#pragma unroll
    for (int t = 16; t < 32; ++t) {
      if (t >= kMaxPlanes || !any_lane_active(left > 0)) break;
      const int b = 31 - t;
      encode_plane<NW>((b >> 3) ? h[b & 7] >> 16 : h[b & 7] & 0xFFFFu, expand, W, n, left);
    }
  }
  zc::shift_right<NW>(W, (uint32_t)(32 * NW - Traits<RATE>::kBlockBits) + left);
  W[0] |= E;
}

// ---- inverse -----------------------------------------------------------------------------

// Negabinary words in coefficient order -> the block's fixed-point values, row-major.
ZC_DEV void inverse_transform(uint32_t (&u)[16], int32_t (&q)[16]) {
#pragma unroll
  for (int c = 0; c < 16; ++c) q[kOrder.v[c]] = zc::negabinary_to_int(u[c]);
#pragma unroll
  for (int c = 0; c < 4; ++c) zc::inverse_lift(q[c], q[4 + c], q[8 + c], q[12 + c]);
#pragma unroll
  for (int r = 0; r < 4; ++r) zc::inverse_lift(q[4 * r], q[4 * r + 1], q[4 * r + 2], q[4 * r + 3]);
}

// Fixed-point values -> fp32: int -> fp32 rounds to nearest even, the scaling by
// 2^(E - 127 - 27) is exact and rounds once more only for subnormal results.
ZC_DEV void scale_block(const int32_t (&q)[16], uint32_t E, float (&out)[16]) {
  const int ex = (int)E - 127 - kFractionBits;
#pragma unroll
  for (int i = 0; i < 16; ++i) out[i] = __builtin_ldexpf((float)q[i], ex);
}

// sum += the block's fp32 values, for exponent bytes where the scaling is exact and finite
// (see scaling_is_exact): the product of the rounded integer and the power of two is then the
// decoded value itself, and the fused multiply-add rounds the sum once, as the addition would.
ZC_DEV void accumulate_scaled(const int32_t (&q)[16], uint32_t E, float (&sum)[16]) {
  const float scale = __builtin_ldexpf(1.0f, (int)E - 127 - kFractionBits);
#pragma unroll
  for (int i = 0; i < 16; ++i) sum[i] = __builtin_fmaf((float)q[i], scale, sum[i]);
}

// Nonzero values have magnitude 1 .. 2^31 before scaling: from E = 28 on none of them becomes
// subnormal, up to E = 250 none overflows.  In the zero block (E = 0) all values are zero, and
// zero times anything finite added to the sum is the sum plus zero.
ZC_DEV bool scaling_is_exact(uint32_t E) { return E - 28u <= 222u || E == 0u; }

// One plane of the embedded code, read from the bottom of the window W.  Returns the
// plane's bit of each coefficient.  n: how many leading coefficients are significant.
//
// The group tests are read in steps that all lanes of the wavefront take together.  A step
// looks the next bits up in the token table (see there for the state s and the rows); if in
// every lane that still reads this plane the entry's tokens lie inside the budget, the step is
// just the entry applied: lanes whose plane is closed read empty entries, lanes out of budget
// apply nothing.  Otherwise (some lane's first token is longer than the look-ahead, or its
// budget ends inside the entry's bits) the step takes the general form: per lane the entry if
// it fits, else one token by count-trailing-zeros with the limits applied.  Budgets of the
// lanes of a wavefront end within a few steps of each other, so the general form is needed
// near a block's end only.  any_lane_active.lanes(p) is the set of lanes where p holds, taken
// per comparison (a compare instruction's result is that set), and .some(set) whether a set
// is non-empty.
template <int NW, class AnyActive>
ZC_DEV uint32_t decode_plane(const uint32_t* token, uint32_t (&W)[NW], uint32_t& n, uint32_t& left,
                             AnyActive any_lane_active) {
  const uint32_t vlen = umin(n, left);
  uint32_t pat = W[0] & ((1u << vlen) - 1u);
  zc::shift_out<NW>(W, vlen);
  left -= vlen;
  uint32_t s = n;   // n = 16: nothing left to test, the plane counts as closed
  for (;;) {
    const bool open = s < kTokenIdleState, funded = left > 0u;
    const auto reading = any_lane_active.lanes(open) & any_lane_active.lanes(funded);
    if (!any_lane_active.some(reading)) break;
    // byte offset of the entry: (clamped state - first row's state) rows, then the next bits;
    // the constant rides on the masking of the bits (it has none of their positions set)
    constexpr uint32_t kRowBytesLg = kLookahead + 2;
    constexpr uint32_t kBias = 0u - (kTokenFirstRowState << kRowBytesLg);
    const uint32_t clamped = umin(umax(s, kTokenFirstRowState), kTokenIdleState);
    uint32_t bits = W[0] & ((1u << kLookahead) - 1u);
    zc::materialise(bits);   // (a bit-field extract, then shift-and-or with the constant, then shift-and-add:
    bits = bits << 2 | kBias;   //  otherwise the constant comes back as an addition of its own)
    zc::materialise(bits);
    const uint32_t at = (clamped << kRowBytesLg) + bits;
    const uint32_t e = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(token) + at);
    const bool unfit = (e >> 20) > left;
    if (!any_lane_active.some(reading & any_lane_active.lanes(unfit))) {
      const uint32_t a = funded ? e : 0u;
      pat |= (a & 0x3FFu) << (s & 31u);
      s += (a >> 10) & 0x3Fu;
      const uint32_t used = (a >> 20) & 15u;
      zc::shift_out<NW>(W, used);
      left -= used;
    } else if (open && funded) {
      // one token with the limits applied where the entry does not fit (its group bit is a one,
      // or the table would have served): zeros up to the one; the run ends at the last
      // coefficient or at the budget.  (The entry is taken up afresh here, so that nothing of
      // this rare form is computed ahead of the branch.)
      uint32_t f = e;
      zc::materialise(f);
      const bool cut = (f >> 20) > left;
      const uint32_t room = umin(15u - s, left - 1u);
      const uint32_t z = umin(count_trailing_zeros(W[0] >> 1), room);
      const uint32_t used = cut ? 1u + z + (z < room ? 1u : 0u) : (f >> 20) & 15u;
      pat |= (cut ? 1u << z : f & 0x3FFu) << s;
      s += cut ? z + 1u : (f >> 10) & 0x3Fu;
      zc::shift_out<NW>(W, used);
      left -= used;
    }
  }
  n = s & 31u;
  return pat;
}

// Whole block up to the fixed-point values; returns the exponent byte.
template <int RATE, class AnyActive>
ZC_DEV uint32_t decode_block_fixed(uint32_t (&W)[Traits<RATE>::kWords], const uint32_t* token, int32_t (&q)[16],
                                   AnyActive any_lane_active) {
  constexpr int NW = Traits<RATE>::kWords;
  constexpr int kPayload = Traits<RATE>::kPayloadBits;
  constexpr int kMaxPlanes = kPayload < 32 ? kPayload : 32;
  const uint32_t E = W[0] & 0xFFu;
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
    lead -= 8u;
  }
  lead = umin(lead, (uint32_t)kPayload);
  uint32_t left = (uint32_t)kPayload - lead;
  if (E == 0u || (kPayload > 32 && lead >= 32u)) left = 0u;
  // past the header byte and the leading zeros: two shifts of less than 32 each (with 32 and
  // more leading zeros nothing is read from the window, whatever it holds)
  zc::shift_out<NW>(W, 8u);
  zc::shift_out<NW>(W, lead & 31u);
  // a lane whose planes start more than 16 below the top (and that has any to read)
  const bool low_start = lead > 16u && left > 0u;
  uint32_t n = 0;
  uint32_t h[8], u[16];
#pragma unroll
  for (int w = 0; w < 8; ++w) h[w] = 0u;
#pragma unroll
  for (int t = 0; t < 16; ++t) {
    if (t >= kMaxPlanes || !any_lane_active(left > 0)) break;
    const int b = 15 - t;
    h[b & 7] |= decode_plane<NW>(token, W, n, left, any_lane_active) << (16 * (b >> 3));
  }
  transpose_halves<true>(h);
#pragma unroll
  for (int w = 0; w < 8; ++w) zc::materialise(h[w]);   // one transpose, not one per half
  const bool deeper = kMaxPlanes > 16 && any_lane_active(left > 0);
  if (!deeper && !any_lane_active(low_start)) {
    // the usual case: at most 16 planes were read and they start within the top 16, so each
    // coefficient is its 16-bit pattern moved up (a lane that read nothing has zero patterns)
    const uint32_t up = (16u - lead) & 31u;
#pragma unroll
    for (int w = 0; w < 8; ++w) {
      u[w] = (h[w] & 0xFFFFu) << up;
      u[w + 8] = (h[w] >> 16) << up;
    }
  } else {
#pragma unroll
    for (int w = 0; w < 8; ++w) {
      u[w] = h[w] << 16;
      u[w + 8] = h[w] & 0xFFFF0000u;
    }
    if (deeper) {
#pragma unroll
      for (int w = 0; w < 8; ++w) h[w] = 0u;
#pragma unroll
      for (int t = 16; t < 32; ++t) {
        if (t >= kMaxPlanes || !any_lane_active(left > 0)) break;
        const int b = 31 - t;
        h[b & 7] |= decode_plane<NW>(token, W, n, left, any_lane_active) << (16 * (b >> 3));
      }
      transpose_halves<true>(h);
#pragma unroll
      for (int w = 0; w < 8; ++w) {
        zc::materialise(h[w]);
        u[w] |= h[w] & 0xFFFFu;
        u[w + 8] |= h[w] >> 16;
      }
    }
#pragma unroll
    for (int c = 0; c < 16; ++c) u[c] >>= (lead & 31u);   // nothing was decoded if lead >= 32
  }
  inverse_transform(u, q);
  return E;
}

template <int RATE, class AnyActive>
ZC_DEV void decode_block(uint32_t (&W)[Traits<RATE>::kWords], const uint32_t* token, float (&out)[16],
                         AnyActive any_lane_active) {
  int32_t q[16];
  const uint32_t E = decode_block_fixed<RATE>(W, token, q, any_lane_active);
  scale_block(q, E, out);
}

}  // namespace zc2d
#endif  // ZC2D_CODEC_H
