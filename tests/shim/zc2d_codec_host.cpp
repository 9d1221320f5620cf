// Host build of the per-block 4 x 4 codec that the GPU kernels run (csrc/zc2d_codec.h),
// for checking its logic on the CPU against the reference.  Test-only.
#include <cstring>

#include "../../paper_2409_02423_amd/csrc/zc2d_codec.h"

namespace {
auto always = [](bool p) { return p; };
constexpr zc2d::ExpandTable kExpand = zc2d::build_expand_table();
constexpr zc2d::TokenTable kToken = zc2d::build_token_table();

template <int RATE>
void enc(const float* x, uint8_t* out) {
  uint32_t b[16], W[zc2d::Traits<RATE>::kWords];
  std::memcpy(b, x, 64);
  zc2d::encode_block<RATE>(b, kExpand.v, W, always);
  std::memcpy(out, W, zc2d::Traits<RATE>::kBlockBytes);
}
template <int RATE>
void dec(const uint8_t* in, float* x) {
  uint32_t W[zc2d::Traits<RATE>::kWords];
  std::memcpy(W, in, zc2d::Traits<RATE>::kBlockBytes);
  float o[16];
  zc2d::decode_block<RATE>(W, kToken.v, o, always);
  std::memcpy(x, o, 64);
}
}  // namespace

extern "C" int zc2d_host_encode_blocks(int rate, const float* x, size_t blocks, uint8_t* out) {
  for (size_t j = 0; j < blocks; ++j) switch (rate) {
      case 2: enc<2>(x + 16 * j, out + j * 4); break;
      case 4: enc<4>(x + 16 * j, out + j * 8); break;
      case 8: enc<8>(x + 16 * j, out + j * 16); break;
      case 16: enc<16>(x + 16 * j, out + j * 32); break;
      default: return -2;
    }
  return 0;
}

extern "C" int zc2d_host_decode_blocks(int rate, const uint8_t* in, size_t blocks, float* x) {
  for (size_t j = 0; j < blocks; ++j) switch (rate) {
      case 2: dec<2>(in + j * 4, x + 16 * j); break;
      case 4: dec<4>(in + j * 8, x + 16 * j); break;
      case 8: dec<8>(in + j * 16, x + 16 * j); break;
      case 16: dec<16>(in + j * 32, x + 16 * j); break;
      default: return -2;
    }
  return 0;
}
