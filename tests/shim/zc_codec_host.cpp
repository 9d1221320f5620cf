// Host build of the per-block codec that the GPU kernels run (csrc/zc_codec.h), so
// that its logic can be checked on the CPU against the reference codec and under
// host sanitizers before it runs on a GPU.  Test-only: the library never runs this.
#include <condition_variable>
#include <cstring>
#include <mutex>
#include <thread>
#include <vector>

#include "../../paper_2409_02423_amd/csrc/zc_codec.h"

namespace {
const zc::EncTable kEnc = zc::build_enc_table();
const zc::DecTable kDec = zc::build_dec_table();
const zc::Dec4Table kDec4 = zc::build_dec4_table();
alignas(4) const zc::Enc4Table kEnc4 = zc::build_enc4_table();
const zc::Dec4HalfTable kDec4Half = zc::build_dec4_half_table();
const zc::Tables kTables = {kEnc.v, kDec.v, kDec4.v, kDec4Half.v};
const zc::Tables kTables4 = {reinterpret_cast<const uint32_t*>(kEnc4.v), kDec.v, kDec4.v, kDec4Half.v};
// one lane alone: the set of lanes where p holds is p itself
struct Alone {
  bool lanes(bool p) const { return p; }
  bool some(bool set) const { return set; }
  bool operator()(bool p) const { return p; }
};
const Alone always;

template <int RATE>
void enc(const float* x, uint8_t* out) {
  uint32_t b[4], W[zc::Traits<RATE>::kWords];
  std::memcpy(b, x, 16);
  zc::encode_block<RATE>(b, RATE == 4 ? kTables4 : kTables, W, always);
  std::memcpy(out, W, zc::Traits<RATE>::kBlockBytes);
}
template <int RATE>
void dec(const uint8_t* in, float* x) {
  uint32_t W[zc::Traits<RATE>::kWords] = {};
  std::memcpy(W, in, zc::Traits<RATE>::kBlockBytes);
  float o[4];
  zc::decode_block<RATE>(W, kTables, o, always);
  std::memcpy(x, o, 16);
}

// A wavefront on the host: `lanes` threads run the per-lane codec in lockstep, and the
// wavefront-wide "does any lane ..." of the kernels is a vote among them.  This is how the
// kernels take their loop decisions, so lanes whose blocks need different numbers of steps
// are exercised together, as on the GPU.
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
  constexpr int B = zc::Traits<RATE>::kBlockBytes;
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
          uint32_t b[4] = {0, 0, 0, 0}, W[zc::Traits<RATE>::kWords];
          if (real) std::memcpy(b, in + 16 * j, 16);
          zc::encode_block<RATE>(b, RATE == 4 ? kTables4 : kTables, W, vote);
          if (real) std::memcpy(out + j * B, W, B);
        } else {
          uint32_t W[zc::Traits<RATE>::kWords] = {};
          if (real) std::memcpy(W, in + j * B, B);
          float o[4];
          zc::decode_block<RATE>(W, kTables, o, vote);
          if (real) std::memcpy(out + 16 * j, o, 16);
        }
      }
    });
  for (auto& th : pool) th.join();
}
}  // namespace

#define ZC_FOR_RATES(F) F(4) F(8) F(12) F(16) F(20) F(24) F(28) F(32)

extern "C" int zc_host_encode_blocks(int rate, const float* x, size_t blocks, uint8_t* out) {
  for (size_t j = 0; j < blocks; ++j) switch (rate) {
#define F(R) case R: enc<R>(x + 4 * j, out + j * (R / 2)); break;
      ZC_FOR_RATES(F)
#undef F
      default: return -2;
    }
  return 0;
}

extern "C" int zc_host_decode_blocks(int rate, const uint8_t* in, size_t blocks, float* x) {
  for (size_t j = 0; j < blocks; ++j) switch (rate) {
#define F(R) case R: dec<R>(in + j * (R / 2), x + 4 * j); break;
      ZC_FOR_RATES(F)
#undef F
      default: return -2;
    }
  return 0;
}

// The same with `lanes` blocks coded in lockstep (see Ballot).
extern "C" int zc_host_encode_wave(int rate, const float* x, size_t blocks, uint8_t* out, int lanes) {
  switch (rate) {
#define F(R) case R: wave<R>(true, reinterpret_cast<const uint8_t*>(x), blocks, out, lanes); break;
    ZC_FOR_RATES(F)
#undef F
    default: return -2;
  }
  return 0;
}

extern "C" int zc_host_decode_wave(int rate, const uint8_t* in, size_t blocks, float* x, int lanes) {
  switch (rate) {
#define F(R) case R: wave<R>(false, in, blocks, reinterpret_cast<uint8_t*>(x), lanes); break;
    ZC_FOR_RATES(F)
#undef F
    default: return -2;
  }
  return 0;
}

// The decompress kernels' tile order (see region_order in zc_codec.h), for a check that it is a
// permutation of the tiles.
extern "C" size_t zc_host_region_order(size_t v, size_t tiles, int lg) {
  return zc::region_order(v, zc::region_bulk(tiles, lg), lg);
}

// Rate 4 in the fused reduce: for each of the 65536 two-byte blocks W0, sum[W0] = (first) or
// sum[W0] += (otherwise) the decoded block, in the form the reduce kernel picks for it (plain
// unless unusual4 says otherwise; `form` 1 forces the plain form, 2 the careful one).
// unusual[W0] receives unusual4's answer.
extern "C" void zc_host_accumulate4_all(int first, int form, float* sum, uint8_t* unusual) {
  for (uint32_t W0 = 0; W0 < 65536u; ++W0) {
    float s[4];
    std::memcpy(s, sum + 4 * W0, 16);
    const bool odd = zc::unusual4(W0);
    unusual[W0] = odd;
    const bool careful = form == 2 || (form == 0 && odd);
    if (careful) {
      if (first) zc::accumulate_careful4<true>(W0, kTables, s);
      else zc::accumulate_careful4<false>(W0, kTables, s);
    } else {
      if (first) zc::accumulate_plain4<true>(W0, kTables, s);
      else zc::accumulate_plain4<false>(W0, kTables, s);
    }
    std::memcpy(sum + 4 * W0, s, 16);
  }
}
