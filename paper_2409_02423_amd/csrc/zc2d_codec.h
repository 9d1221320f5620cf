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
//   * the 16 coefficient words are bit-transposed (two 16 x 16 transposes done at once
//     in the two halves of 32-bit registers), so that plane k is one 16-bit pattern;
//     the patterns are parked in a per-lane column of LDS, from which the plane loop
//     (uniform over the wavefront) fetches one pattern per step;
//   * within a plane the newly significant coefficients are found with count-trailing-
//     zeros instead of bit by bit: each costs a group bit, its run of zeros and (unless
//     it is the last coefficient) a one;
//   * a budget cut inside a run places the decoded one after the zeros read so far,
//     which is the lowest index still possible.
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

// ---- 16 x 16 bit transpose in both halves of sixteen 32-bit words --------------------
// In: word c, bit b (b < 16) and bit 16 + b.  Out: word b, bit c = in word c bit b, and
// bit 16 + c = in word c bit 16 + b.  Four rounds of block swaps between word pairs.
ZC_DEV constexpr void transpose16(uint32_t (&a)[16]) {
  constexpr uint32_t mask[4] = {0x00FF00FFu, 0x0F0F0F0Fu, 0x33333333u, 0x55555555u};
  int m = 0;
#pragma unroll
  for (int j = 8; j >= 1; j >>= 1, ++m)
#pragma unroll
    for (int r = 0; r < 16; ++r)
      if ((r & j) == 0) {
        const uint32_t lo = a[r], hi = a[r + j];
        a[r] = (lo & mask[m]) | ((hi & mask[m]) << j);
        a[r + j] = ((lo >> j) & mask[m]) | (hi & ~mask[m]);
      }
}

namespace selfcheck {
constexpr bool transpose_ok() {
  uint32_t a[16] = {}, ref[16] = {};
  uint32_t s = 0x9E3779B9u;
  for (int c = 0; c < 16; ++c) { s = s * 1664525u + 1013904223u; a[c] = s; }
  for (int c = 0; c < 16; ++c)
    for (int b = 0; b < 16; ++b) {
      ref[b] |= ((a[c] >> b) & 1u) << c;
      ref[b] |= ((a[c] >> (16 + b)) & 1u) << (16 + c);
    }
  transpose16(a);
  for (int c = 0; c < 16; ++c)
    if (a[c] != ref[c]) return false;
  return true;
}
static_assert(transpose_ok(), "16 x 16 bit transpose");
}  // namespace selfcheck

// Per-lane column of sixteen 32-bit rows in LDS: row r of lane l at plane_rows[r * stride + l].
struct PlaneStore {
  uint32_t* rows;   // already offset to this lane
  int stride;       // lanes per row
};

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
  uint32_t m = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i) m = umax(m, x[i] & 0x7FFFFFFFu);
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

template <int RATE, class AnyActive>
ZC_DEV void encode_block(const uint32_t (&x)[16], PlaneStore lds, uint32_t (&W)[Traits<RATE>::kWords],
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
  for (int c = 0; c < 16; ++c) u[c] <<= (lead & 31u);   // top plane to bit 31
  transpose16(u);   // u[r]: plane r in the low half, plane 16 + r in the high half
#pragma unroll
  for (int r = 0; r < 16; ++r) lds.rows[r * lds.stride] = u[r];
#pragma unroll
  for (int j = 0; j < NW; ++j) W[j] = 0;
  uint32_t n = 0;
#pragma unroll 1
  for (int t = 0; t < kMaxPlanes; ++t) {
    if (!any_lane_active(left > 0)) break;
    const int k = 31 - t;
    const uint32_t row = lds.rows[(k & 15) * lds.stride];
    const uint32_t pat = (k & 16) ? row >> 16 : row & 0xFFFFu;
    // coefficients already significant: their bits as they are
    const uint32_t vlen = umin(n, left);
    zc::shift_in<NW>(W, pat, vlen);
    left -= vlen;
    // the rest: one group test per newly significant coefficient
    uint32_t rest = pat >> n, i = n, code = 0, len = 0;
    while (any_lane_active(rest != 0u)) {
      if (rest != 0u) {
        const uint32_t z = count_trailing_zeros(rest);
        code |= 1u << len;   // the group holds a one
        len += 1u + z;       // z zeros on the way to it
        if (i + z < 15u) {   // the one itself, unless it is the last coefficient
          code |= 1u << len;
          len += 1u;
        }
        rest >>= z + 1u;
        i += z + 1u;
      }
    }
    if (i < 16u) len += 1u;  // the closing group bit 0
    const uint32_t glen = umin(len, left);
    zc::shift_in<NW>(W, code, glen);
    left -= glen;
    n = i;
  }
  zc::shift_right<NW>(W, (uint32_t)(32 * NW - Traits<RATE>::kBlockBits) + left);
  W[0] |= E;
}

// ---- inverse -----------------------------------------------------------------------------

ZC_DEV void inverse_transform(uint32_t (&u)[16], uint32_t E, float (&out)[16]) {
  int32_t q[16];
#pragma unroll
  for (int c = 0; c < 16; ++c) q[kOrder.v[c]] = zc::from_negabinary(u[c]);
#pragma unroll
  for (int c = 0; c < 4; ++c) zc::inverse_lift(q[c], q[4 + c], q[8 + c], q[12 + c]);
#pragma unroll
  for (int r = 0; r < 4; ++r) zc::inverse_lift(q[4 * r], q[4 * r + 1], q[4 * r + 2], q[4 * r + 3]);
  const int ex = (int)E - 127 - kFractionBits;
#pragma unroll
  for (int i = 0; i < 16; ++i) out[i] = __builtin_ldexpf((float)q[i], ex);
}

template <int RATE, class AnyActive>
ZC_DEV void decode_block(uint32_t (&W)[Traits<RATE>::kWords], PlaneStore lds, float (&out)[16],
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
  zc::shift_right<NW>(W, lead + 8u);
#pragma unroll
  for (int r = 0; r < 16; ++r) lds.rows[r * lds.stride] = 0u;
  uint32_t n = 0;
#pragma unroll 1
  for (int t = 0; t < kMaxPlanes; ++t) {
    if (!any_lane_active(left > 0)) break;
    const uint32_t vlen = umin(n, left);
    uint32_t pat = W[0] & ((1u << vlen) - 1u);
    zc::shift_out<NW>(W, vlen);
    left -= vlen;
    uint32_t i = n;
    bool open = true;
    while (any_lane_active(open && i < 16u && left > 0u)) {
      uint32_t used = 0;
      if (open && i < 16u && left > 0u) {
        const uint32_t group = W[0] & 1u;
        used = 1u;
        if (!group) {
          open = false;
        } else {
          // zeros up to the one; the run ends at the last coefficient or at the budget
          const uint32_t room = umin(15u - i, left - 1u);
          const uint32_t z = umin(count_trailing_zeros(W[0] >> 1), room);
          used += z + (z < room ? 1u : 0u);
          i += z;
          pat |= 1u << i;
          i += 1u;
        }
      }
      zc::shift_out<NW>(W, used);
      left -= used;
    }
    n = i;
    const int k = 31 - t;
    uint32_t* row = lds.rows + (k & 15) * lds.stride;
    *row |= (k & 16) ? pat << 16 : pat;
  }
  uint32_t u[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) u[r] = lds.rows[r * lds.stride];
  transpose16(u);
#pragma unroll
  for (int c = 0; c < 16; ++c) u[c] >>= (lead & 31u);   // nothing was decoded if lead >= 32
  inverse_transform(u, E, out);
}

}  // namespace zc2d
#endif  // ZC2D_CODEC_H
