// zc_half.h -- bf16 / fp16 message values on the device: exact widening to fp32 and
// rounding back to the nearest half-precision value, ties to even (the paper does not state
// its message precision; see the half-precision calls in include/zc.h).
#ifndef ZC_HALF_H
#define ZC_HALF_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

// Element types of a message buffer (values of enum zc_dtype).
constexpr int kF32 = 0, kBF16 = 1, kF16 = 2;

// Exact widening of a bf16 / fp16 bit pattern to an fp32 bit pattern.
template <int DT>
__device__ __forceinline__ uint32_t widen_half(uint32_t h) {
  if constexpr (DT == kBF16) {
    return h << 16;
  } else {
    const _Float16 v = __builtin_bit_cast(_Float16, (uint16_t)h);
    return __float_as_uint((float)v);
  }
}

// Nearest bf16 / fp16, ties to even.  bf16: add 0x7FFF plus the lowest kept bit to the
// fp32 pattern and drop 16 bits; a carry into the exponent is the next binade or infinity.
template <int DT>
__device__ __forceinline__ uint32_t narrow_half(float f) {
  if constexpr (DT == kBF16) {
    const uint32_t b = __float_as_uint(f);
    return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
  } else {
    return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)f);
  }
}

}  // namespace
#endif  // ZC_HALF_H
