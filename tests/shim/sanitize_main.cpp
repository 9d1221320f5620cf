// Driver for a host build with -fsanitize=address,undefined: runs the reference codecs
// (oracle/*.c) and the host builds of the kernels' per-lane codecs (tests/shim/*_host.cpp)
// over arbitrary bytes, edge values, ragged shapes and damaged lossless streams, and
// compares the two sides where both exist.  Test-only; exits non-zero on any mismatch
// (the sanitizers abort on their own findings).
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

extern "C" {
size_t zc_ref_compressed_size(size_t n, int rate);
int zc_ref_compress(const float* in, size_t n, int rate, void* out, size_t out_cap);
int zc_ref_decompress(const void* in, size_t n, int rate, float* out);
int zc_ref_reduce_compressed(const void* const* in, int k, size_t n, int rate, void* out, size_t out_cap);
int zc_ref_reduce_mixed(const void* const* in, int k, const float* local, size_t n, int rate, void* out, size_t out_cap);
int zc_ref_reduce_decompress(const void* const* in, int k, const float* local, size_t n, int rate, float* out);
int zc_ref_compress_half(const uint16_t* in, int dtype, size_t n, int rate, void* out, size_t out_cap);
int zc_ref_decompress_half(const void* in, size_t n, int rate, int dtype, uint16_t* out);
size_t zc2d_ref_compressed_size(size_t rows, size_t cols, int rate);
int zc2d_ref_compress(const float* in, size_t rows, size_t cols, int rate, void* out, size_t out_cap);
int zc2d_ref_decompress(const void* in, size_t rows, size_t cols, int rate, float* out);
int zc2d_ref_reduce_mixed(const void* const* in, int k, const float* local, size_t rows, size_t cols, int rate, void* out,
                          size_t out_cap);
size_t zl_ref_max_compressed_size(size_t n);
int zl_ref_compress(const uint32_t* in, size_t n, void* out, size_t out_cap, size_t* out_bytes);
int zl_ref_decompress(const void* in, size_t in_bytes, size_t n, uint32_t* out);
int zc_host_encode_blocks(int rate, const float* x, size_t blocks, uint8_t* out);
int zc_host_decode_blocks(int rate, const uint8_t* in, size_t blocks, float* x);
int zc2d_host_encode_blocks(int rate, const float* x, size_t blocks, uint8_t* out);
int zc2d_host_decode_blocks(int rate, const uint8_t* in, size_t blocks, float* x);
void zl_host_to_planes(const uint32_t* words, size_t groups, uint32_t* references, uint32_t* bitmaps, uint32_t* planes);
void zl_host_from_planes(const uint32_t* planes, const uint32_t* references, size_t groups, uint32_t* words);
}

static uint64_t g_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd() {
  g_state ^= g_state << 13; g_state ^= g_state >> 7; g_state ^= g_state << 17;
  return (uint32_t)(g_state >> 16);
}
static int g_failed = 0;
#define CHECK(cond, ...) do { if (!(cond)) { std::fprintf(stderr, "MISMATCH: " __VA_ARGS__); std::fprintf(stderr, "\n"); ++g_failed; } } while (0)

// finite fp32 bit patterns over the whole exponent range, with zeros, subnormals and shared magnitudes mixed in
static void fill_values(std::vector<float>& x) {
  for (size_t i = 0; i < x.size(); ++i) {
    uint32_t b = rnd();
    const uint32_t kind = rnd() % 8;
    if (kind == 0) b = 0;
    else if (kind == 1) b &= 0x807FFFFFu;                                  // subnormal
    else if (kind == 2 && i) { uint32_t p; std::memcpy(&p, &x[i - 1], 4); b = (b & 0x807FFFFFu) | (p & 0x7F800000u); }
    if (((b >> 23) & 0xFF) >= 254) b = (b & 0x807FFFFFu) | (100u << 23);  // keep below 2^127
    std::memcpy(&x[i], &b, 4);
  }
}

int main() {
  // ---- blocks of 4 ----
  for (int rate = 4; rate <= 32; rate += 4) {
    const size_t blocks = 3000, n = 4 * blocks, size = zc_ref_compressed_size(n, rate);
    std::vector<uint8_t> s[3];
    for (auto& v : s) { v.resize(size); for (auto& b : v) b = (uint8_t)rnd(); }
    for (size_t i = 0; i < size / 2; ++i) s[1][i] &= (uint8_t)rnd();
    std::vector<float> a(n), b(n), local(n);
    CHECK(zc_ref_decompress(s[0].data(), n, rate, a.data()) == 0, "decompress rc rate %d", rate);
    CHECK(zc_host_decode_blocks(rate, s[0].data(), blocks, b.data()) == 0, "host decode rc rate %d", rate);
    CHECK(std::memcmp(a.data(), b.data(), 4 * n) == 0, "arbitrary bytes decode differently at rate %d", rate);
    fill_values(local);
    const void* in[3] = {s[0].data(), s[1].data(), s[2].data()};
    std::vector<uint8_t> out(size);
    CHECK(zc_ref_reduce_compressed(in, 3, n, rate, out.data(), size) == 0, "reduce rc");
    CHECK(zc_ref_reduce_mixed(in, 2, local.data(), n - 1, rate, out.data(), size) == 0, "reduce_mixed rc");
    CHECK(zc_ref_reduce_decompress(in, 3, local.data(), n - 3, rate, a.data()) == 0, "reduce_decompress rc");
    // values -> stream on both sides
    std::vector<float> x(n);
    fill_values(x);
    std::vector<uint8_t> c0(size), c1(size);
    CHECK(zc_ref_compress(x.data(), n, rate, c0.data(), size) == 0, "compress rc");
    CHECK(zc_host_encode_blocks(rate, x.data(), blocks, c1.data()) == 0, "host encode rc");
    CHECK(c0 == c1, "edge values encode differently at rate %d", rate);
    for (size_t cut = 1; cut <= 3; ++cut) {   // ragged tails write exactly their size
      const size_t m = n - cut, sz = zc_ref_compressed_size(m, rate);
      std::vector<uint8_t> c(sz);
      std::vector<float> y(m);
      CHECK(zc_ref_compress(x.data(), m, rate, c.data(), sz) == 0 && zc_ref_decompress(c.data(), m, rate, y.data()) == 0, "ragged rc");
    }
    std::vector<uint16_t> h(n), hb(n);
    for (auto& v : h) { v = (uint16_t)rnd(); if (((v >> 7) & 0xFF) == 0xFF) v &= 0x807F; }
    CHECK(zc_ref_compress_half(h.data(), 1, n, rate, c0.data(), size) == 0, "compress_half rc");
    CHECK(zc_ref_decompress_half(s[2].data(), n, rate, 2, hb.data()) == 0, "decompress_half rc");
  }
  // ---- blocks of 4 x 4 ----
  for (int rate : {2, 4, 8, 16}) {
    const size_t rows = 64, cols = 96, blocks = rows * cols / 16, size = zc2d_ref_compressed_size(rows, cols, rate);
    std::vector<uint8_t> s(size), t(size);
    for (auto& b : s) b = (uint8_t)rnd();
    for (auto& b : t) b = (uint8_t)(rnd() & rnd());
    std::vector<float> a(rows * cols), b(rows * cols), blk(rows * cols);
    CHECK(zc2d_ref_decompress(s.data(), rows, cols, rate, a.data()) == 0, "2d decompress rc");
    CHECK(zc2d_host_decode_blocks(rate, s.data(), blocks, blk.data()) == 0, "2d host decode rc");
    for (size_t bi = 0; bi < rows / 4; ++bi)      // the host codec works block by block: put the blocks back in place
      for (size_t bj = 0; bj < cols / 4; ++bj)
        for (int r = 0; r < 4; ++r)
          for (int c = 0; c < 4; ++c) b[(4 * bi + r) * cols + 4 * bj + c] = blk[16 * (bi * (cols / 4) + bj) + 4 * r + c];
    CHECK(std::memcmp(a.data(), b.data(), 4 * a.size()) == 0, "2d arbitrary bytes decode differently at rate %d", rate);
    std::vector<float> x(rows * cols);
    fill_values(x);
    for (auto shape : {std::pair<size_t, size_t>{64, 96}, {5, 7}, {1, 1}, {3, 96}, {64, 2}}) {
      const size_t sz = zc2d_ref_compressed_size(shape.first, shape.second, rate);
      std::vector<uint8_t> c(sz), o(sz);
      std::vector<float> y(shape.first * shape.second);
      CHECK(zc2d_ref_compress(x.data(), shape.first, shape.second, rate, c.data(), sz) == 0, "2d compress rc");
      CHECK(zc2d_ref_decompress(c.data(), shape.first, shape.second, rate, y.data()) == 0, "2d decompress rc");
      const void* in[2] = {c.data(), s.data()};
      if (sz <= size)
        CHECK(zc2d_ref_reduce_mixed(in, 2, x.data(), shape.first, shape.second, rate, o.data(), sz) == 0, "2d reduce rc");
    }
    std::vector<uint8_t> c0(size), c1(size);
    std::vector<float> xb(rows * cols);
    for (size_t bi = 0; bi < rows / 4; ++bi)
      for (size_t bj = 0; bj < cols / 4; ++bj)
        for (int r = 0; r < 4; ++r)
          for (int c = 0; c < 4; ++c) xb[16 * (bi * (cols / 4) + bj) + 4 * r + c] = x[(4 * bi + r) * cols + 4 * bj + c];
    CHECK(zc2d_ref_compress(x.data(), rows, cols, rate, c0.data(), size) == 0, "2d compress rc");
    CHECK(zc2d_host_encode_blocks(rate, xb.data(), blocks, c1.data()) == 0, "2d host encode rc");
    CHECK(c0 == c1, "2d edge values encode differently at rate %d", rate);
  }
  // ---- lossless ----
  for (size_t n : {(size_t)1, (size_t)8191, (size_t)8192, (size_t)20000}) {
    std::vector<uint32_t> w(n), back(n);
    for (size_t i = 0; i < n; ++i) w[i] = (rnd() % 4 == 0) ? rnd() : (0x3F000000u | (rnd() & 0x007FFFFFu));
    const size_t cap = zl_ref_max_compressed_size(n);
    std::vector<uint8_t> s(cap);
    size_t bytes = 0;
    CHECK(zl_ref_compress(w.data(), n, s.data(), cap, &bytes) == 0 && bytes <= cap, "lossless compress rc");
    CHECK(zl_ref_decompress(s.data(), bytes, n, back.data()) == 0 && back == w, "lossless round trip");
    for (int trial = 0; trial < 200; ++trial) {   // damaged streams are rejected or decoded, never read out of bounds
      std::vector<uint8_t> d(s.begin(), s.begin() + bytes);
      const int hits = 1 + (int)(rnd() % 4);
      for (int hit = 0; hit < hits; ++hit) d[rnd() % (trial % 2 ? (bytes < 64 ? bytes : 64) : bytes)] = (uint8_t)rnd();
      const size_t given = trial % 5 == 0 ? (size_t)(rnd() % (bytes + 1)) : bytes;
      (void)zl_ref_decompress(d.data(), given, n, back.data());
    }
  }
  {
    const size_t groups = 300;
    std::vector<uint32_t> w(32 * groups), refs(groups), maps(groups), planes(32 * groups), back(32 * groups);
    for (auto& v : w) v = rnd() & (rnd() | 0xFF000000u);
    zl_host_to_planes(w.data(), groups, refs.data(), maps.data(), planes.data());
    zl_host_from_planes(planes.data(), refs.data(), groups, back.data());
    CHECK(back == w, "lossless per-lane round trip");
  }
  if (g_failed) return 1;
  std::puts("sanitize driver: ok");
  return 0;
}
