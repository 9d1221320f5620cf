// Host build of the per-block 4 x 4 codec that the GPU kernels run (csrc/zc2d_codec.h),
// for checking its logic on the CPU against the reference.  Test-only.
#include <condition_variable>
#include <cstring>
#include <mutex>
#include <thread>
#include <vector>

#include "../../paper_2409_02423_amd/csrc/zc2d_codec.h"

namespace {
// one lane alone: the set of lanes where p holds is p itself
struct Alone {
  bool lanes(bool p) const { return p; }
  bool some(bool set) const { return set; }
  bool operator()(bool p) const { return p; }
};
const Alone always;
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

// A wavefront on the host: `lanes` threads run the per-lane codec in lockstep and take the
// kernels' wavefront-wide votes among themselves (as in zc_codec_host.cpp).
struct Ballot {
  explicit Ballot(int n) : lanes(n) {}
  bool vote(bool p) {
    std::unique_lock<std::mutex> lock(mu);
    any = any || p;
    if (++arrived == lanes) {
      result = any;
      any = false;
      arrived = 0;
      ++round;
      cv.notify_all();
      return result;
    }
    const unsigned long mine = round;
    cv.wait(lock, [&] { return round != mine; });
    return result;
  }
  std::mutex mu;
  std::condition_variable cv;
  int lanes, arrived = 0;
  bool any = false, result = false;
  unsigned long round = 0;
};

template <int RATE>
void wave(bool encode, const uint8_t* in, size_t blocks, uint8_t* out, int lanes) {
  constexpr int B = zc2d::Traits<RATE>::kBlockBytes;
  Ballot ballot(lanes);
  // a thread's share of a set of lanes is its own predicate; the vote joins them
  struct Vote {
    Ballot* b;
    bool lanes(bool p) const { return p; }
    bool some(bool set) const { return b->vote(set); }
    bool operator()(bool p) const { return b->vote(p); }
  };
  const Vote vote{&ballot};
  const size_t waves = (blocks + lanes - 1) / lanes;
  std::vector<std::thread> pool;
  for (int t = 0; t < lanes; ++t)
    pool.emplace_back([&, t] {
      for (size_t w = 0; w < waves; ++w) {
        const size_t j = w * lanes + t;
        const bool real = j < blocks;   // lanes past the end code a zero block and drop the result
        if (encode) {
          uint32_t b[16] = {}, W[zc2d::Traits<RATE>::kWords];
          if (real) std::memcpy(b, in + 64 * j, 64);
          zc2d::encode_block<RATE>(b, kExpand.v, W, vote);
          if (real) std::memcpy(out + j * B, W, B);
        } else {
          uint32_t W[zc2d::Traits<RATE>::kWords] = {};
          if (real) std::memcpy(W, in + j * B, B);
          float o[16];
          zc2d::decode_block<RATE>(W, kToken.v, o, vote);
          if (real) std::memcpy(out + 64 * j, o, 64);
        }
      }
    });
  for (auto& th : pool) th.join();
}
}  // namespace

extern "C" int zc2d_host_wave(int rate, int encode, const void* in, size_t blocks, void* out, int lanes) {
  const uint8_t* src = static_cast<const uint8_t*>(in);
  uint8_t* dst = static_cast<uint8_t*>(out);
  switch (rate) {
    case 2: wave<2>(encode != 0, src, blocks, dst, lanes); break;
    case 4: wave<4>(encode != 0, src, blocks, dst, lanes); break;
    case 8: wave<8>(encode != 0, src, blocks, dst, lanes); break;
    case 16: wave<16>(encode != 0, src, blocks, dst, lanes); break;
    default: return -2;
  }
  return 0;
}

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
