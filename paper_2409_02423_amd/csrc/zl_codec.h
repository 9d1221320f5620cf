// zl_codec.h -- per-lane pieces of the lossless codec ("ZL-1"), as run by one GPU lane.
//
// The paper's first hybrid scheme sends model-parallel traffic through a lossless codec
// of the MPC kind (Sec. II-A, Sec. III-A); this is the format built for that role: a
// lane owns one group of 32 words of a chunk (four consecutive words from each of its
// eight 16-byte reads), describes each by its distance from the group's largest
// magnitude, bit-transposes the 32 residuals in registers and keeps the non-zero planes.
#ifndef ZL_CODEC_H
#define ZL_CODEC_H

#include <stdint.h>

#if defined(__HIPCC__)
#define ZL_DEV __host__ __device__ __forceinline__
#else
#define ZL_DEV inline
#endif

namespace zl {

constexpr uint32_t kMagic = 0x31304C5Au;   // "ZL01"
constexpr int kChunkWords = 8192;
constexpr int kGroups = 256;               // groups per chunk = lanes per workgroup
constexpr int kHeaderBytes = 32;
constexpr int kFixedChunkBytes = 8 * kGroups;   // references and bitmaps

// Table entry: two state bits above a 62-bit byte count.
constexpr uint64_t kValueMask = ((uint64_t)1 << 62) - 1;
constexpr uint64_t kOwnSize = (uint64_t)1 << 62;   // while compressing: the chunk's own size
constexpr uint64_t kEnd = (uint64_t)2 << 62;       // final: where the chunk ends in the payload

// 32 x 32 bit transpose: out word k, bit j = in word j, bit k.  Its own inverse.
ZL_DEV constexpr void transpose32(uint32_t (&a)[32]) {
  constexpr uint32_t mask[5] = {0x0000FFFFu, 0x00FF00FFu, 0x0F0F0F0Fu, 0x33333333u, 0x55555555u};
  int m = 0;
#pragma unroll
  for (int s = 16; s >= 1; s >>= 1, ++m)
#pragma unroll
    for (int i = 0; i < 32; ++i)
      if ((i & s) == 0) {
        const uint32_t lo = a[i], hi = a[i + s];
        a[i] = (lo & mask[m]) | ((hi & mask[m]) << s);
        a[i + s] = ((lo >> s) & mask[m]) | (hi & ~mask[m]);
      }
}

namespace selfcheck {
constexpr bool transpose_ok() {
  uint32_t a[32] = {}, ref[32] = {};
  uint32_t s = 0x2545F491u;
  for (int j = 0; j < 32; ++j) { s = s * 1664525u + 1013904223u; a[j] = s; }
  for (int j = 0; j < 32; ++j)
    for (int k = 0; k < 32; ++k) ref[k] |= ((a[j] >> k) & 1u) << j;
  transpose32(a);
  for (int k = 0; k < 32; ++k)
    if (a[k] != ref[k]) return false;
  return true;
}
static_assert(transpose_ok(), "32 x 32 bit transpose");
}  // namespace selfcheck

// Words of a group -> its reference (largest magnitude as a bit pattern), and in place
// the planes of the residuals sign | (reference - magnitude).  Returns the bitmap of
// non-zero planes.
ZL_DEV uint32_t to_planes(uint32_t (&w)[32], uint32_t& reference) {
  uint32_t m = 0;
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    const uint32_t mag = w[j] & 0x7FFFFFFFu;
    m = mag > m ? mag : m;
  }
#pragma unroll
  for (int j = 0; j < 32; ++j) w[j] = (w[j] & 0x80000000u) | (m - (w[j] & 0x7FFFFFFFu));
  transpose32(w);
  uint32_t bitmap = 0;
#pragma unroll
  for (int k = 0; k < 32; ++k) bitmap |= (w[k] != 0u ? 1u : 0u) << k;
  reference = m;
  return bitmap;
}

// Planes (absent ones as zero) and reference -> the words, in place.  The distance wraps
// within 31 bits, so residuals that no encoder produces still decode.
ZL_DEV void from_planes(uint32_t (&p)[32], uint32_t reference) {
  transpose32(p);
#pragma unroll
  for (int j = 0; j < 32; ++j) p[j] = (p[j] & 0x80000000u) | ((reference - (p[j] & 0x7FFFFFFFu)) & 0x7FFFFFFFu);
}

}  // namespace zl
#endif  // ZL_CODEC_H
