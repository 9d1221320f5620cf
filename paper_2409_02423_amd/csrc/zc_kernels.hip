// zc_kernels.hip -- gfx950 kernels and the C ABI of libzc (see include/zc.h).
//
// Three streaming kernels, one lane per block of 4 values, grid-stride over the
// buffer.  All are specialised per rate.  Each lane reads 16 contiguous bytes of
// fp32 (compress) or RATE/2 contiguous bytes of stream (decompress, reduce), so a
// wavefront touches one contiguous span per access; the code tables are staged in
// LDS once per workgroup; the next block is fetched before the current one is
// coded.  No matrix cores: nothing here is a contraction.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include "../../include/zc.h"
#include "zc_codec.h"
#include "zc_half.h"

namespace {

// staged into LDS with 16-byte loads
__device__ __align__(16) const zc::EncTable g_enc_table = zc::build_enc_table();
__device__ __align__(16) const zc::DecTable g_dec_table = zc::build_dec_table();
__device__ __align__(16) const zc::Dec4Table g_dec4_table = zc::build_dec4_table();
__device__ __align__(16) const zc::Dec4HalfTable g_dec4_half_table = zc::build_dec4_half_table();
__device__ __align__(16) const zc::Enc4Table g_enc4_table = zc::build_enc4_table();

constexpr int kThreads = 256;          // 4 wavefronts
constexpr int kEncWords = zc::kEncPlaneEntries + 256;
constexpr int kDecWords = zc::kDecPlaneEntries + 256;
constexpr int kDec4Words = 256 * 4;
constexpr int kDec4HalfWords = 256 * 2;
constexpr int kEnc4Words = (1 << 13) / 4;
constexpr int kMaxChunks = 16;
constexpr size_t kWideBlocks = 512;     // blocks per wavefront and pass of the wide rate-4 kernels

// The wavefront-wide votes of the codec: lanes(p) is the set of lanes where p holds (taken
// per comparison, so that the compare instruction's own mask is the set and sets combine on
// the scalar side), some(set) whether it is non-empty; any_lane_active(p) = some(lanes(p)).
struct AnyLane {
  __device__ uint64_t lanes(bool p) const { return __builtin_amdgcn_ballot_w64(p); }
  __device__ bool some(uint64_t set) const { return set != 0; }
  __device__ bool operator()(bool p) const { return __builtin_amdgcn_ballot_w64(p) != 0; }
};

// Copy a code table into LDS, 16 bytes per lane and step.
template <int WORDS>
__device__ __forceinline__ void stage_table(uint32_t* lds, const uint32_t* table) {
  static_assert(WORDS % 4 == 0, "table size");
  constexpr int kVecs = WORDS / 4;
  constexpr int kPerThread = (kVecs + kThreads - 1) / kThreads;
  uint4 v[kPerThread];
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    int idx = threadIdx.x + i * kThreads;
    v[i] = reinterpret_cast<const uint4*>(table)[idx < kVecs ? idx : 0];
  }
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    int idx = threadIdx.x + i * kThreads;
    if (idx < kVecs) reinterpret_cast<uint4*>(lds)[idx] = v[i];
  }
}

// The same in two parts, for the fused reduce, which needs two or three tables: every lane issues
// all of its loads of all of them back to back before it writes, one wait instead of one per step (as
// the compiler schedules the function above).  That made the reduce kernels 1 to 3 % faster
// and the decompress kernels, which live on memory rate, 2 to 3 % slower, so only the former
// use it.  In a last, partial step the lanes beyond the table's end copy its first entry once more.
template <int WORDS>
struct TableCopy {
  static_assert(WORDS % 4 == 0, "table size");
  static constexpr int kVecs = WORDS / 4;
  static constexpr int kSteps = (kVecs + kThreads - 1) / kThreads;
  uint4 v[kSteps];
  int idx[kSteps];
  __device__ __forceinline__ explicit TableCopy(const uint32_t* table) {
#pragma unroll
    for (int i = 0; i < kSteps; ++i) {
      idx[i] = threadIdx.x + i * kThreads;
      if ((i + 1) * kThreads > kVecs && idx[i] >= kVecs) idx[i] = 0;
      v[i] = reinterpret_cast<const uint4*>(table)[idx[i]];
    }
  }
  __device__ __forceinline__ void put(uint32_t* lds) const {
#pragma unroll
    for (int i = 0; i < kSteps; ++i) reinterpret_cast<uint4*>(lds)[idx[i]] = v[i];
  }
};

// Rate 4 encodes its one payload byte with one look-up in the 8192-entry table; the other
// rates use the two-planes-per-step table.
template <int RATE>
constexpr int encoder_table_words() { return RATE == 4 ? kEnc4Words : kEncWords; }
template <int RATE>
__device__ __forceinline__ const uint32_t* encoder_table() {
  if constexpr (RATE == 4) return reinterpret_cast<const uint32_t*>(g_enc4_table.v);
  else return g_enc_table.v;
}

// Rate 4 decodes its one payload byte with the 256-entry block table; the other rates
// use the per-plane table.
template <int RATE>
constexpr int decoder_table_words() { return RATE == 4 ? kDec4Words : kDecWords; }
template <int RATE>
__device__ __forceinline__ const uint32_t* decoder_table() {
  if constexpr (RATE == 4) return reinterpret_cast<const uint32_t*>(g_dec4_table.v);
  else return g_dec_table.v;
}

template <int RATE>
__device__ __forceinline__ zc::Tables decoder_tables(const uint32_t* dec, const uint32_t* enc, const uint32_t* dec_half = nullptr) {
  if constexpr (RATE == 4) return zc::Tables{enc, nullptr, reinterpret_cast<const float*>(dec), reinterpret_cast<const uint16_t*>(dec_half)};
  else return zc::Tables{enc, dec, nullptr, nullptr};
}

template <int RATE>
__device__ __forceinline__ void stage_encoder_table(uint32_t* lds) {
  stage_table<encoder_table_words<RATE>()>(lds, encoder_table<RATE>());
}

template <int RATE>
__device__ __forceinline__ zc::Tables stage_decoder_table(uint32_t* lds, const uint32_t* enc) {
  stage_table<decoder_table_words<RATE>()>(lds, decoder_table<RATE>());
  return decoder_tables<RATE>(lds, enc);
}

// All tables of the fused reduce: the decoder's (at rate 4 also its half-precision copy) and,
// unless the sum is stored as fp32, the encoder's.
template <int RATE, bool ENCODER>
__device__ __forceinline__ zc::Tables stage_reduce_tables(uint32_t* dec, uint32_t* dec_half, uint32_t* enc) {
  using Dec = TableCopy<decoder_table_words<RATE>()>;
  using Half = TableCopy<RATE == 4 ? kDec4HalfWords : 4>;
  using Enc = TableCopy<ENCODER ? encoder_table_words<RATE>() : 4>;
  constexpr int kSteps = Dec::kSteps + (RATE == 4 ? Half::kSteps : 0) + (ENCODER ? Enc::kSteps : 0);
  const Dec d(decoder_table<RATE>());
  const Half h(RATE == 4 ? reinterpret_cast<const uint32_t*>(g_dec4_half_table.v) : decoder_table<RATE>());
  const Enc e(ENCODER ? encoder_table<RATE>() : decoder_table<RATE>());
  d.put(dec);
  if constexpr (RATE == 4) h.put(dec_half);
  if constexpr (ENCODER) e.put(enc);
  __builtin_amdgcn_sched_group_barrier(0x020, kSteps, 0);   // (for the instruction scheduler: the loads first,
  __builtin_amdgcn_sched_group_barrier(0x200, kSteps, 0);   // then the LDS writes)
  return decoder_tables<RATE>(dec, enc, dec_half);
}

// ---- block I/O ----------------------------------------------------------------------

// Message buffers are streamed once.  Measured on MI355X: non-temporal 16-byte fp32
// loads and stores are faster than plain ones (the decompress kernel's 1 GiB of
// output by a third).  The narrow compressed stream is read with non-temporal loads as well
// (see load_stream; the rate-4 decompress kernel that takes 16 bytes per lane uses a plain
// load) and written with non-temporal stores by the compress kernels and plain ones by the
// fused reduce (see store_stream).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <class T>
__device__ __forceinline__ T nt_load(const T* p) { return __builtin_nontemporal_load(p); }

template <class T>
__device__ __forceinline__ void nt_store(T* p, T v) { __builtin_nontemporal_store(v, p); }

// Stores of the compressed stream are plain: the stream is small and is read again
// soon (by the next kernel of a ring hop, or by the network), so it may stay cached.
template <class T>
__device__ __forceinline__ void stream_store(T* p, T v) { *p = v; }

// Four values of block j as fp32 bit patterns.
template <int DT>
__device__ __forceinline__ void load_values(const void* in, size_t j, uint32_t (&x)[4]) {
  if constexpr (DT == kF32) {
    u32x4 v = nt_load(reinterpret_cast<const u32x4*>(in) + j);
    x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
  } else {
    u32x2 v = nt_load(reinterpret_cast<const u32x2*>(in) + j);
    x[0] = widen_half<DT>(v.x & 0xFFFFu); x[1] = widen_half<DT>(v.x >> 16);
    x[2] = widen_half<DT>(v.y & 0xFFFFu); x[3] = widen_half<DT>(v.y >> 16);
  }
}

// The ragged last block (n % 4 values) repeats the last value.
template <int DT>
__device__ __forceinline__ void load_values_ragged(const void* in, size_t n, uint32_t (&x)[4]) {
  const size_t base = n & ~(size_t)3;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const size_t idx = base + i < n ? base + i : n - 1;
    if constexpr (DT == kF32) x[i] = reinterpret_cast<const uint32_t*>(in)[idx];
    else x[i] = widen_half<DT>(reinterpret_cast<const uint16_t*>(in)[idx]);
  }
}

template <int DT>
__device__ __forceinline__ void store_values(void* out, size_t j, const float (&x)[4]) {
  if constexpr (DT == kF32) {
    u32x4 v = {__float_as_uint(x[0]), __float_as_uint(x[1]), __float_as_uint(x[2]), __float_as_uint(x[3])};
    nt_store(reinterpret_cast<u32x4*>(out) + j, v);
  } else {
    u32x2 v = {narrow_half<DT>(x[0]) | narrow_half<DT>(x[1]) << 16, narrow_half<DT>(x[2]) | narrow_half<DT>(x[3]) << 16};
    nt_store(reinterpret_cast<u32x2*>(out) + j, v);
  }
}

template <int DT>
__device__ __forceinline__ void store_values_ragged(void* out, size_t n, const float (&x)[4]) {
  const size_t base = n & ~(size_t)3;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (base + i < n) {
      if constexpr (DT == kF32) reinterpret_cast<float*>(out)[base + i] = x[i];
      else reinterpret_cast<uint16_t*>(out)[base + i] = (uint16_t)narrow_half<DT>(x[i]);
    }
}

// Compressed block j: RATE/2 bytes at byte j*RATE/2; bits beyond the block are zero.
// Non-temporal loads: a stream is read once, and keeping the reduce's inputs out of the
// last-level cache leaves its output there for the decompress kernel that follows (in the
// compress, reduce, decompress step on 2^28 values at rate 4 that kernel went from 0.210 to
// 0.176 ms, what it takes when launched back to back).
template <int RATE>
__device__ __forceinline__ void load_stream(const uint8_t* in, size_t j, uint32_t (&W)[zc::Traits<RATE>::kWords]) {
  constexpr int B = zc::Traits<RATE>::kBlockBytes;
  const uint8_t* p = in + j * B;
  if constexpr (B == 16) {
    u32x4 v = nt_load(reinterpret_cast<const u32x4*>(p));
    W[0] = v.x; W[1] = v.y; W[2] = v.z; W[3] = v.w;
  } else if constexpr (B == 8) {
    u32x2 v = nt_load(reinterpret_cast<const u32x2*>(p));
    W[0] = v.x; W[1] = v.y;
  } else if constexpr (B % 4 == 0) {
#pragma unroll
    for (int i = 0; i < B / 4; ++i) W[i] = nt_load(reinterpret_cast<const uint32_t*>(p) + i);
  } else {
    const uint16_t* h = reinterpret_cast<const uint16_t*>(p);
#pragma unroll
    for (int i = 0; i < zc::Traits<RATE>::kWords; ++i) W[i] = 0;
#pragma unroll
    for (int i = 0; i < B / 2; ++i) W[i / 2] |= (uint32_t)nt_load(h + i) << (16 * (i % 2));
  }
}

// NT: non-temporal stores (the compress kernels: their stream is read next by another
// device or a later kernel, and not keeping it in the caches made them 6 to 8 % faster);
// plain stores otherwise (the fused reduce, whose output the next hop reads at once).
template <int RATE, bool NT = false>
__device__ __forceinline__ void store_stream(uint8_t* out, size_t j, const uint32_t (&W)[zc::Traits<RATE>::kWords]) {
  constexpr int B = zc::Traits<RATE>::kBlockBytes;
  uint8_t* p = out + j * B;
  auto put = [](auto* q, auto v) {
    if constexpr (NT) nt_store(q, v);
    else stream_store(q, v);
  };
  if constexpr (B == 16) {
    u32x4 v = {W[0], W[1], W[2], W[3]};
    put(reinterpret_cast<u32x4*>(p), v);
  } else if constexpr (B == 8) {
    u32x2 v = {W[0], W[1]};
    put(reinterpret_cast<u32x2*>(p), v);
  } else if constexpr (B % 4 == 0) {
#pragma unroll
    for (int i = 0; i < B / 4; ++i) put(reinterpret_cast<uint32_t*>(p) + i, W[i]);
  } else {
    uint16_t* h = reinterpret_cast<uint16_t*>(p);
#pragma unroll
    for (int i = 0; i < B / 2; ++i) put(h + i, (uint16_t)(W[i / 2] >> (16 * (i % 2))));
  }
}

// ---- kernels ------------------------------------------------------------------------
// Work is cut into tiles of U * 256 consecutive blocks; a workgroup takes tiles with a
// grid stride and lane t codes blocks t, t + 256, ... of the tile, so every access of
// a wavefront is one contiguous span.  All U loads of the next tile are issued before
// the current tile is coded (under a test that is the same for the whole workgroup; a
// workgroup's last tile fetches nothing more): that keeps U accesses per lane in flight,
// which is what the narrow stream accesses (RATE/2 bytes per lane) need to cover memory
// latency.  Blocks after the
// last whole tile are coded one per lane, and the ragged last block (n % 4 values) by
// a single lane.

// Blocks per lane and tile, from measurements on MI355X: the rate-4 compress and
// decompress kernels have so little work per block that one block per lane is fastest;
// the others gain from four accesses in flight per lane, except the fused reduce above
// rate 4, which is bound by its arithmetic and runs 2 to 6 % faster with two (fewer
// registers, more wavefronts per SIMD).
template <int RATE> constexpr int compress_unroll() { return RATE == 4 ? 1 : 4; }
template <int RATE> constexpr int decompress_unroll() { return RATE == 4 ? 1 : 4; }
template <int RATE> constexpr int reduce_unroll() { return RATE == 4 ? 4 : 2; }

template <int RATE, int U, int DT>
__global__ __launch_bounds__(kThreads) void compress_kernel(const void* __restrict__ in, size_t n,
                                                            uint8_t* __restrict__ out) {
  __shared__ __align__(16) uint32_t enc[encoder_table_words<RATE>()];
  stage_encoder_table<RATE>(enc);
  __syncthreads();
  const zc::Tables tab = {enc, nullptr, nullptr};
  constexpr int NW = zc::Traits<RATE>::kWords;
  constexpr size_t kTile = (size_t)U * kThreads;
  const size_t whole = n / 4;
  const size_t tiles = whole / kTile;   // below 2^30 (n is at most 2^40): tile numbers compare as 32-bit values, on the scalar side
  size_t t = blockIdx.x;
  if (t < tiles) {
    uint32_t x[U][4];
#pragma unroll
    for (int u = 0; u < U; ++u) load_values<DT>(in, t * kTile + u * kThreads + threadIdx.x, x[u]);
    while (true) {
      const size_t tn = t + gridDim.x;
      const bool more = (uint32_t)tn < (uint32_t)tiles;   // the same in every lane of the workgroup
      uint32_t xn[U][4];
      if (more) {
#pragma unroll
        for (int u = 0; u < U; ++u) load_values<DT>(in, tn * kTile + u * kThreads + threadIdx.x, xn[u]);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        uint32_t W[NW];
        zc::encode_block<RATE>(x[u], tab, W, AnyLane());
        store_stream<RATE, (RATE != 12)>(out, t * kTile + u * kThreads + threadIdx.x, W);   // (rate 12, three 2-byte stores per block: plain stores measured 9 % faster)
      }
      if (!more) break;
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int i = 0; i < 4; ++i) x[u][i] = xn[u][i];
      t = tn;
    }
  }
  for (size_t j = tiles * kTile + (size_t)blockIdx.x * kThreads + threadIdx.x; j < whole;
       j += (size_t)gridDim.x * kThreads) {
    uint32_t x[4], W[NW];
    load_values<DT>(in, j, x);
    zc::encode_block<RATE>(x, tab, W, AnyLane());
    store_stream<RATE, true>(out, j, W);
  }
  if ((n & 3) != 0 && blockIdx.x == 0 && threadIdx.x == 0) {
    uint32_t x[4], W[NW];
    load_values_ragged<DT>(in, n, x);
    zc::encode_block<RATE>(x, tab, W, AnyLane());
    store_stream<RATE, true>(out, whole, W);
  }
}

template <int RATE, int U, int DT>
__global__ __launch_bounds__(kThreads) void decompress_kernel(const uint8_t* __restrict__ in, size_t n,
                                                              void* __restrict__ out) {
  __shared__ __align__(16) uint32_t dec[decoder_table_words<RATE>()];
  const zc::Tables tab = stage_decoder_table<RATE>(dec, nullptr);
  __syncthreads();
  constexpr int NW = zc::Traits<RATE>::kWords;
  constexpr size_t kTile = (size_t)U * kThreads;
  const size_t whole = n / 4;
  const size_t tiles = whole / kTile;   // below 2^30 (n is at most 2^40): tile numbers compare as 32-bit values, on the scalar side
  size_t t = blockIdx.x;
  if (t < tiles) {
    uint32_t W[U][NW];
#pragma unroll
    for (int u = 0; u < U; ++u) load_stream<RATE>(in, t * kTile + u * kThreads + threadIdx.x, W[u]);
    while (true) {
      const size_t tn = t + gridDim.x;
      const bool more = (uint32_t)tn < (uint32_t)tiles;   // the same in every lane of the workgroup
      uint32_t Wn[U][NW];
      if (more) {
#pragma unroll
        for (int u = 0; u < U; ++u) load_stream<RATE>(in, tn * kTile + u * kThreads + threadIdx.x, Wn[u]);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float y[4];
        zc::decode_block<RATE>(W[u], tab, y, AnyLane());
        store_values<DT>(out, t * kTile + u * kThreads + threadIdx.x, y);
      }
      if (!more) break;
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int i = 0; i < NW; ++i) W[u][i] = Wn[u][i];
      t = tn;
    }
  }
  for (size_t j = tiles * kTile + (size_t)blockIdx.x * kThreads + threadIdx.x; j < whole;
       j += (size_t)gridDim.x * kThreads) {
    uint32_t W[NW];
    float y[4];
    load_stream<RATE>(in, j, W);
    zc::decode_block<RATE>(W, tab, y, AnyLane());
    store_values<DT>(out, j, y);
  }
  if ((n & 3) != 0 && blockIdx.x == 0 && threadIdx.x == 0) {
    uint32_t W[NW];
    float y[4];
    load_stream<RATE>(in, whole, W);
    zc::decode_block<RATE>(W, tab, y, AnyLane());
    store_values_ragged<DT>(out, n, y);
  }
}

// Rate 4: a block's stream is two bytes, so a lane that stores its own block's moves 128
// bytes per wavefront and access.  Here a wavefront codes 512 consecutive blocks (lane,
// lane + 64, ...: contiguous loads), collects their streams in 1 KiB of LDS of its own and
// writes them with one 16-byte store per lane (compress<4> 0.222 -> 0.213 ms on 2^28 values).
template <int DT>
__global__ __launch_bounds__(kThreads) void compress4_wide_kernel(const void* __restrict__ in, size_t wave_tiles,
                                                                  uint8_t* __restrict__ out) {
  __shared__ __align__(16) uint32_t enc[encoder_table_words<4>()];
  __shared__ __align__(16) uint32_t stage[kThreads / 64][256];
  stage_encoder_table<4>(enc);
  __syncthreads();
  const zc::Tables tab = {enc, nullptr, nullptr};
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // a workgroup's four wave tiles are neighbours (32 KiB of fp32 input); these groups of four
  // are taken in region order, 1 MiB of input per region, as in the decompress kernel below
  // (a kernel without arithmetic that reads and writes the same way: 0.1945 ms in plain order,
  // 0.188 ms with regions of 1 or 2 MiB)
  constexpr int kRegionLg = 5;
  const size_t groups = wave_tiles / (kThreads / 64), bulk = zc::region_bulk(groups, kRegionLg);
  auto wave_tile = [&](size_t g) { return g < groups ? zc::region_order(g, bulk, kRegionLg) * (kThreads / 64) + wave : g * (kThreads / 64) + wave; };
  size_t g = blockIdx.x;
  size_t t = wave_tile(g);
  if (t >= wave_tiles) return;
  uint32_t x[8][4];
#pragma unroll
  for (int r = 0; r < 8; ++r) load_values<DT>(in, t * 512 + 64 * r + lane, x[r]);
  for (;;) {
    const size_t gn = g + gridDim.x;
    const size_t tn = wave_tile(gn);
    const bool more = tn < wave_tiles;
    const size_t next = (more ? tn : t) * 512 + lane;
    uint32_t xn[8][4];
#pragma unroll
    for (int r = 0; r < 8; ++r) load_values<DT>(in, next + 64 * r, xn[r]);
    uint16_t* halves = reinterpret_cast<uint16_t*>(stage[wave]);
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      uint32_t W[1];
      zc::encode_block<4>(x[r], tab, W, AnyLane());
      halves[64 * r + lane] = (uint16_t)W[0];
    }
    __builtin_amdgcn_wave_barrier();
    const u32x4 v = reinterpret_cast<const u32x4*>(stage[wave])[lane];
    *reinterpret_cast<u32x4*>(out + t * 1024 + 16 * lane) = v;
    __builtin_amdgcn_wave_barrier();
    if (!more) break;
#pragma unroll
    for (int r = 0; r < 8; ++r)
#pragma unroll
      for (int i = 0; i < 4; ++i) x[r][i] = xn[r][i];
    t = tn;
    g = gn;
  }
}

// The same the other way round: a wavefront fetches the streams of 512 consecutive blocks
// in one 16-byte access per lane, passes them through 1 KiB of LDS of its own and decodes
// blocks lane, lane + 64, ... so that its stores stay contiguous (decompress<4> 0.227 ->
// 0.214 ms on 2^28 values).
template <int DT>
__global__ __launch_bounds__(kThreads) void decompress4_wide_kernel(const uint8_t* __restrict__ in, size_t wave_tiles,
                                                                    void* __restrict__ out) {
  __shared__ __align__(16) uint32_t dec[kDec4Words];
  __shared__ __align__(16) uint32_t stage[kThreads / 64][256];
  const zc::Tables tab = stage_decoder_table<4>(dec, nullptr);
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // a workgroup's four wave tiles are neighbours (32 KiB of fp32 output); these groups of four
  // are taken in region order, 1 MiB of output per region
  constexpr int kRegionLg = 5;
  const size_t groups = wave_tiles / (kThreads / 64), bulk = zc::region_bulk(groups, kRegionLg);
  auto wave_tile = [&](size_t g) { return g < groups ? zc::region_order(g, bulk, kRegionLg) * (kThreads / 64) + wave : g * (kThreads / 64) + wave; };
  size_t g = blockIdx.x;
  size_t t = wave_tile(g);
  if (t >= wave_tiles) return;
  u32x4 v = *reinterpret_cast<const u32x4*>(in + t * 1024 + 16 * lane);
  for (;;) {
    const size_t gn = g + gridDim.x;
    const size_t tn = wave_tile(gn);
    const bool more = tn < wave_tiles;
    u32x4 vn = v;
    if (more) vn = *reinterpret_cast<const u32x4*>(in + tn * 1024 + 16 * lane);
    reinterpret_cast<u32x4*>(stage[wave])[lane] = v;
    __builtin_amdgcn_wave_barrier();
    const uint16_t* halves = reinterpret_cast<const uint16_t*>(stage[wave]);
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      uint32_t W[1] = {halves[64 * r + lane]};
      float y[4];
      zc::decode_block<4>(W, tab, y, AnyLane());
      store_values<DT>(out, t * 512 + 64 * r + lane, y);
    }
    __builtin_amdgcn_wave_barrier();
    if (!more) break;
    v = vn;
    t = tn;
    g = gn;
  }
}

struct ChunkPointers {
  const uint8_t* p[kMaxChunks];
};

// The fused reduce.  Decode block j of every chunk, add in fp32 in chunk order, add
// the raw local values last if there are any (LOCAL), then either encode the sum or
// store it as fp32 (RAW_OUT).  Nothing but the inputs and the output touches memory.
// The output may be one of the inputs of the same kind: a lane reads its blocks of all
// inputs before it writes them, and no other lane touches those blocks.  Tiles are
// visited chunk by chunk, (tile, chunk 0), (tile, chunk 1), ..., (next tile, chunk 0),
// and the next one in that order is fetched before the current one is decoded; the
// local values of a tile are requested before its first chunk is decoded.
template <int RATE, int U, bool LOCAL, bool RAW_OUT, int K>
__global__ __launch_bounds__(kThreads) void reduce_kernel(ChunkPointers chunks, int k_given, const float* local, size_t n,
                                                          uint8_t* out, float* out_raw) {
  const int k = K > 0 ? K : k_given;   // K > 0: the number of chunks is known when the kernel is compiled
  __shared__ __align__(16) uint32_t dec[decoder_table_words<RATE>()];
  __shared__ __align__(16) uint32_t dec_half[RATE == 4 ? kDec4HalfWords : 4];
  __shared__ __align__(16) uint32_t enc[RAW_OUT ? 4 : encoder_table_words<RATE>()];
  const zc::Tables tab = stage_reduce_tables<RATE, !RAW_OUT>(dec, dec_half, enc);
  __syncthreads();
  constexpr int NW = zc::Traits<RATE>::kWords;
  constexpr size_t kTile = (size_t)U * kThreads;
  const size_t whole = n / 4;
  const size_t tiles = whole / kTile;   // below 2^30 (n is at most 2^40): tile numbers compare as 32-bit values, on the scalar side

  // s: the sum of one block; finishes it (local add, then encode or store)
  auto finish = [&](float (&s)[4], const uint32_t (&loc)[4], size_t j) {
    if constexpr (LOCAL) {
#pragma unroll
      for (int i = 0; i < 4; ++i) s[i] += __uint_as_float(loc[i]);
    }
    if constexpr (RAW_OUT) {
      store_values<kF32>(out_raw, j, s);
    } else {
      uint32_t x[4], Wo[NW];
#pragma unroll
      for (int i = 0; i < 4; ++i) x[i] = __float_as_uint(s[i]);
      zc::encode_block<RATE>(x, tab, Wo, AnyLane());
      store_stream<RATE>(out, j, Wo);
    }
  };

  size_t t = blockIdx.x;
  if constexpr (K == 0) {
    // Any number of chunks: a tile's blocks are asked for from up to kGroup chunks at once and
    // summed as they arrive, so that a tile waits for memory once per group and not once per
    // chunk (with one chunk fetched ahead of the one being summed, the 8-way reduce of 2^25
    // values took 0.203 ms at rate 8 and 0.049 ms at rate 4; so 0.191 and, with the
    // half-precision table, 0.043 ms).
    constexpr int kGroup = NW >= 3 || RATE == 4 ? 4 : 8;
    for (; (uint32_t)t < (uint32_t)tiles; t += gridDim.x) {
      uint32_t loc[U][4];
      if constexpr (LOCAL) {
#pragma unroll
        for (int u = 0; u < U; ++u) load_values<kF32>(local, t * kTile + u * kThreads + threadIdx.x, loc[u]);
      }
      float s[U][4];
      bool unusual = false;
      for (int c0 = 0; c0 < k; c0 += kGroup) {
        uint32_t W[kGroup][U][NW];
#pragma unroll
        for (int g = 0; g < kGroup; ++g) {
          if (c0 + g < k) {
#pragma unroll
            for (int u = 0; u < U; ++u) load_stream<RATE>(chunks.p[c0 + g], t * kTile + u * kThreads + threadIdx.x, W[g][u]);
          }
        }
#pragma unroll
        for (int g = 0; g < kGroup; ++g) {
          if (c0 + g < k) {
            const bool first = g == 0 && c0 == 0;
#pragma unroll
            for (int u = 0; u < U; ++u) {
              if constexpr (RATE == 4) {
                unusual = unusual | zc::unusual4(W[g][u][0]);
                if (first) zc::accumulate_plain4<true>(W[g][u][0], tab, s[u]);
                else zc::accumulate_plain4<false>(W[g][u][0], tab, s[u]);
              } else {
                float y[4];
                zc::decode_block<RATE>(W[g][u], tab, y, AnyLane());
#pragma unroll
                for (int i = 0; i < 4; ++i) s[u][i] = first ? y[i] : s[u][i] + y[i];
              }
            }
          }
        }
      }
      if constexpr (RATE == 4) {
        // (see the two-chunk form below)
        if (AnyLane()(unusual)) {
          for (int c = 0; c < k; ++c) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
              uint32_t Wc[NW];
              load_stream<RATE>(chunks.p[c], t * kTile + u * kThreads + threadIdx.x, Wc);
              if (c == 0) zc::accumulate_careful4<true>(Wc[0], tab, s[u]);
              else zc::accumulate_careful4<false>(Wc[0], tab, s[u]);
            }
          }
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) finish(s[u], loc[u], t * kTile + u * kThreads + threadIdx.x);
    }
  } else if (t < tiles) {
    uint32_t W[U][NW];
#pragma unroll
    for (int u = 0; u < U; ++u) load_stream<RATE>(chunks.p[0], t * kTile + u * kThreads + threadIdx.x, W[u]);
    while (true) {
      const size_t tn = t + gridDim.x;
      const bool more = (uint32_t)tn < (uint32_t)tiles;
      uint32_t loc[U][4];
      if constexpr (LOCAL) {
#pragma unroll
        for (int u = 0; u < U; ++u) load_values<kF32>(local, t * kTile + u * kThreads + threadIdx.x, loc[u]);
      }
      float s[U][4];
      bool unusual = false;
#pragma unroll
      for (int c = 0; c < k; ++c) {
        const bool last = c + 1 == k;
        const uint8_t* src = chunks.p[last ? 0 : c + 1];
        const size_t next = (last ? tn : t) * kTile + threadIdx.x;
        uint32_t Wn[U][NW];
        if (!last || more) {   // after the last chunk of the last tile there is nothing to fetch
#pragma unroll
          for (int u = 0; u < U; ++u) load_stream<RATE>(src, next + u * kThreads, Wn[u]);
        }
        if constexpr (RATE == 4) {
          // rate 4: the plain form for every block, and a note of whether any block was outside
          // what that form covers (the tile is then summed again, see below)
#pragma unroll
          for (int u = 0; u < U; ++u) {
            unusual = unusual | zc::unusual4(W[u][0]);
            if (c == 0) zc::accumulate_plain4<true>(W[u][0], tab, s[u]);
            else zc::accumulate_plain4<false>(W[u][0], tab, s[u]);
          }
        } else {
#pragma unroll
          for (int u = 0; u < U; ++u) {
            float y[4];
            zc::decode_block<RATE>(W[u], tab, y, AnyLane());
#pragma unroll
            for (int i = 0; i < 4; ++i) s[u][i] = c ? s[u][i] + y[i] : y[i];
          }
        }
        if (!last || more) {
#pragma unroll
          for (int u = 0; u < U; ++u)
#pragma unroll
            for (int i = 0; i < NW; ++i) W[u][i] = Wn[u][i];
        }
      }
      if constexpr (RATE == 4) {
        // some block of this tile, in some lane of the wavefront, has a nonzero payload under a
        // zero exponent byte or an exponent byte at which a decoded value may overflow (arbitrary
        // bytes, or values of 2^127 and more): fetch the tile's blocks again (nothing of the tile
        // has been written yet) and sum them in the careful form
        if (AnyLane()(unusual)) {
          for (int c = 0; c < k; ++c) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
              uint32_t Wc[NW];
              load_stream<RATE>(chunks.p[c], t * kTile + u * kThreads + threadIdx.x, Wc);
              if (c == 0) zc::accumulate_careful4<true>(Wc[0], tab, s[u]);
              else zc::accumulate_careful4<false>(Wc[0], tab, s[u]);
            }
          }
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) finish(s[u], loc[u], t * kTile + u * kThreads + threadIdx.x);
      if (!more) break;
      t = tn;
    }
  }

  // sum of one block read directly (blocks after the last whole tile, and the ragged block)
  auto direct_sum = [&](size_t j, float (&s)[4]) {
    for (int c = 0; c < k; ++c) {
      uint32_t W[NW];
      float y[4];
      load_stream<RATE>(chunks.p[c], j, W);
      zc::decode_block<RATE>(W, tab, y, AnyLane());
#pragma unroll
      for (int i = 0; i < 4; ++i) s[i] = c ? s[i] + y[i] : y[i];
    }
  };
  for (size_t j = tiles * kTile + (size_t)blockIdx.x * kThreads + threadIdx.x; j < whole;
       j += (size_t)gridDim.x * kThreads) {
    float s[4] = {0.f, 0.f, 0.f, 0.f};
    uint32_t loc[4] = {0, 0, 0, 0};
    if constexpr (LOCAL) load_values<kF32>(local, j, loc);
    direct_sum(j, s);
    finish(s, loc, j);
  }
  if ((n & 3) != 0 && blockIdx.x == 0 && threadIdx.x == 0) {
    float s[4] = {0.f, 0.f, 0.f, 0.f};
    direct_sum(whole, s);
    if constexpr (LOCAL) {
      uint32_t loc[4];
      load_values_ragged<kF32>(local, n, loc);
#pragma unroll
      for (int i = 0; i < 4; ++i) s[i] += __uint_as_float(loc[i]);
    }
    if constexpr (RAW_OUT) {
      store_values_ragged<kF32>(out_raw, n, s);
    } else {
      // the result is compress(sum): the pad repeats the last valid sum
      const int valid = (int)(n & 3);
      const float pad = valid == 1 ? s[0] : (valid == 2 ? s[1] : s[2]);
      uint32_t x[4], Wo[NW];
#pragma unroll
      for (int i = 0; i < 4; ++i) x[i] = __float_as_uint(i < valid ? s[i] : pad);
      zc::encode_block<RATE>(x, tab, Wo, AnyLane());
      store_stream<RATE>(out, whole, Wo);
    }
  }
}

// ---- host side ----------------------------------------------------------------------

int compute_units() {
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cached[dev] == 0) {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    cached[dev] = cus;
  }
  return cached[dev];
}

// Workgroups per CU in the grid (each loops over tiles with a grid stride).  Eight
// 256-thread workgroups fill a CU; launching several times that lets the dispatcher
// even out the data-dependent coding time and keeps more fetches in flight.  Measured on
// 2^28 values, 16 to 256 per CU: compress and decompress gain up to 128 (rate 8 compress
// 0.252 ms at 32, 0.221 at 128; rate 4 decompress 0.190 at 24, 0.174 at 128) and lose
// again beyond; the decoder at rates 8 and 12 is best near 112; the fused reduce, bound by
// arithmetic, is flat from 32 to 96 and worse outside.
// The library reads no environment variable; only a build with -DZC_TUNING_KNOBS (never
// the shipped one) lets ZC_WORKGROUPS_PER_CU override these numbers for tuning runs.
enum Kernel { kCompress, kDecompress, kReduce, kReduceRaw };   // kReduceRaw: the reduce that stores fp32

int workgroups_per_cu(Kernel kernel, int rate) {
#ifdef ZC_TUNING_KNOBS
  if (const char* e = getenv("ZC_WORKGROUPS_PER_CU")) {
    const int v = atoi(e);
    if (v >= 1 && v <= 1024) return v;
  }
#endif
  switch (kernel) {
    case kCompress: return 128;
    case kDecompress: return rate == 4 || rate >= 16 ? 128 : 112;
    case kReduceRaw: return rate >= 16 ? 128 : 96;   // writes 16 bytes per block: closer to the decoder than to the reduce
    default: return rate == 4 ? 48 : 64;
  }
}

// blocks_per_lane: the kernel's U; a workgroup's unit of work is a tile of U * 256 blocks, and
// no more workgroups are launched than there are tiles (each stages the code tables first:
// a workgroup without a tile would do that for nothing), at least `tiles_each` tiles apiece.
unsigned grid_for(size_t n, Kernel kernel, int rate, int blocks_per_lane) {
  const size_t blocks = (n + 3) / 4, tile = (size_t)blocks_per_lane * kThreads;
  size_t tiles_each = 1;
#ifdef ZC_TUNING_KNOBS
  if (const char* e = getenv("ZC_TILES_EACH")) tiles_each = (size_t)atoi(e) > 0 ? (size_t)atoi(e) : 1;
#endif
  size_t groups = (blocks + tile * tiles_each - 1) / (tile * tiles_each);
  if (groups == 0) groups = 1;
  const size_t cap = (size_t)compute_units() * (size_t)workgroups_per_cu(kernel, rate);
  return (unsigned)(groups < cap ? groups : cap);
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

constexpr size_t kMaxValues = (size_t)1 << 40;

int finish_launch() { return hipGetLastError() == hipSuccess ? ZC_OK : ZC_ERR_LAUNCH; }

}  // namespace

#define ZC_DISPATCH_RATE(rate, CALL) \
  switch (rate) {                    \
    case 4: CALL(4); break;          \
    case 8: CALL(8); break;          \
    case 12: CALL(12); break;        \
    case 16: CALL(16); break;        \
    case 20: CALL(20); break;        \
    case 24: CALL(24); break;        \
    case 28: CALL(28); break;        \
    case 32: CALL(32); break;        \
    default: return ZC_ERR_RATE;     \
  }

extern "C" {

int zc_version(void) { return 100; }

const char* zc_strerror(int code) {
  switch (code) {
    case ZC_OK: return "ok";
    case ZC_ERR_NULL: return "null pointer";
    case ZC_ERR_RATE: return "unsupported rate (a multiple of 4 between 4 and 32; 2, 4, 8 or 16 for the 4 x 4 block codec)";
    case ZC_ERR_SIZE: return "buffer too large";
    case ZC_ERR_CAPACITY: return "output capacity smaller than zc_compressed_size(n, rate)";
    case ZC_ERR_K: return "number of chunks outside [1, 16]";
    case ZC_ERR_ALIGN: return "device pointer not 16-byte aligned";
    case ZC_ERR_LAUNCH: return "kernel launch failed";
    case ZC_ERR_DTYPE: return "dtype must be ZC_BF16 or ZC_F16";
    case ZC_ERR_STREAM: return "not a complete lossless stream";
    default: return "unknown error code";
  }
}

int zc_rate_supported(int rate) { return rate >= 4 && rate <= 32 && rate % 4 == 0; }

int zc_rate_for_class(enum zc_class c) {
  switch (c) {
    case ZC_DP_GRADIENT: return 8;
    case ZC_TP_ACTIVATION:
    case ZC_PP_ACTIVATION:
    case ZC_ZERO_PARAM:
    case ZC_OPT_STATE: return 16;
    default: return 0;
  }
}

int zc_codec_for_class(enum zc_scheme s, enum zc_class c, int* rate) {
  const int fixed = zc_rate_for_class(c);
  if (fixed == 0 || (s != ZC_SCHEME_ZHYBRID && s != ZC_SCHEME_MZHYBRID)) return -1;
  const bool lossless = s == ZC_SCHEME_MZHYBRID && c != ZC_DP_GRADIENT;
  if (rate) *rate = lossless ? 0 : fixed;
  return lossless ? ZC_CODEC_LOSSLESS : ZC_CODEC_FIXED_RATE;
}

size_t zc_compressed_size(size_t n, int rate) {
  if (!zc_rate_supported(rate)) return 0;
  return (n / 4 + (n % 4 ? 1 : 0)) * (size_t)(rate / 2);
}

static int launch_compress(const void* d_in, int dtype, size_t n, int rate, void* d_out, size_t out_cap,
                           void* stream) {
  if (dtype != ZC_F32 && dtype != ZC_BF16 && dtype != ZC_F16) return ZC_ERR_DTYPE;
  if (!zc_rate_supported(rate)) return ZC_ERR_RATE;
  if (n == 0) return ZC_OK;
  if (!d_in || !d_out) return ZC_ERR_NULL;
  if (!aligned16(d_in) || !aligned16(d_out)) return ZC_ERR_ALIGN;
  if (n > kMaxValues) return ZC_ERR_SIZE;
  if (out_cap < zc_compressed_size(n, rate)) return ZC_ERR_CAPACITY;
  hipStream_t s = static_cast<hipStream_t>(stream);
  uint8_t* out = static_cast<uint8_t*>(d_out);
  if (rate == 4 && n / 4 >= kWideBlocks) {
    // whole runs of 512 blocks per wavefront go through the wide kernel, the rest through the general one
    const size_t wave_tiles = (n / 4) / kWideBlocks;
    const size_t groups = (wave_tiles + kThreads / 64 - 1) / (kThreads / 64);
    const size_t cap = (size_t)compute_units() * (size_t)workgroups_per_cu(kCompress, 4);
    const dim3 grid((unsigned)(groups < cap ? groups : cap));
    if (dtype == ZC_F32) hipLaunchKernelGGL(compress4_wide_kernel<kF32>, grid, dim3(kThreads), 0, s, d_in, wave_tiles, out);
    else if (dtype == ZC_BF16) hipLaunchKernelGGL(compress4_wide_kernel<kBF16>, grid, dim3(kThreads), 0, s, d_in, wave_tiles, out);
    else hipLaunchKernelGGL(compress4_wide_kernel<kF16>, grid, dim3(kThreads), 0, s, d_in, wave_tiles, out);
    const size_t done = wave_tiles * kWideBlocks * 4;
    out += done / 2;
    d_in = static_cast<const uint8_t*>(d_in) + done * (dtype == ZC_F32 ? 4 : 2);
    n -= done;
    if (n == 0) return finish_launch();
  }
#define LAUNCH(R, DT)                                                                                            \
  hipLaunchKernelGGL((compress_kernel<R, compress_unroll<R>(), DT>), dim3(grid_for(n, kCompress, R, compress_unroll<R>())), \
                     dim3(kThreads), 0, s, d_in, n, out)
#define CALL(R)                                   \
  do {                                            \
    if (dtype == ZC_F32) LAUNCH(R, kF32);         \
    else if (dtype == ZC_BF16) LAUNCH(R, kBF16);  \
    else LAUNCH(R, kF16);                         \
  } while (0)
  ZC_DISPATCH_RATE(rate, CALL)
#undef CALL
#undef LAUNCH
  return finish_launch();
}

static int launch_decompress(const void* d_in, size_t n, int rate, int dtype, void* d_out, void* stream) {
  if (dtype != ZC_F32 && dtype != ZC_BF16 && dtype != ZC_F16) return ZC_ERR_DTYPE;
  if (!zc_rate_supported(rate)) return ZC_ERR_RATE;
  if (n == 0) return ZC_OK;
  if (!d_in || !d_out) return ZC_ERR_NULL;
  if (!aligned16(d_in) || !aligned16(d_out)) return ZC_ERR_ALIGN;
  if (n > kMaxValues) return ZC_ERR_SIZE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const uint8_t* in = static_cast<const uint8_t*>(d_in);
  if (rate == 4 && n / 4 >= kWideBlocks) {
    const size_t wave_tiles = (n / 4) / kWideBlocks;
    const size_t groups = (wave_tiles + kThreads / 64 - 1) / (kThreads / 64);
    const size_t cap = (size_t)compute_units() * (size_t)workgroups_per_cu(kDecompress, 4);
    const dim3 grid((unsigned)(groups < cap ? groups : cap));
    if (dtype == ZC_F32) hipLaunchKernelGGL(decompress4_wide_kernel<kF32>, grid, dim3(kThreads), 0, s, in, wave_tiles, d_out);
    else if (dtype == ZC_BF16) hipLaunchKernelGGL(decompress4_wide_kernel<kBF16>, grid, dim3(kThreads), 0, s, in, wave_tiles, d_out);
    else hipLaunchKernelGGL(decompress4_wide_kernel<kF16>, grid, dim3(kThreads), 0, s, in, wave_tiles, d_out);
    const size_t done = wave_tiles * kWideBlocks * 4;
    in += done / 2;
    d_out = static_cast<uint8_t*>(d_out) + done * (dtype == ZC_F32 ? 4 : 2);
    n -= done;
    if (n == 0) return finish_launch();
  }
#define LAUNCH(R, DT)                                                                                            \
  hipLaunchKernelGGL((decompress_kernel<R, decompress_unroll<R>(), DT>), dim3(grid_for(n, kDecompress, R, decompress_unroll<R>())), \
                     dim3(kThreads), 0, s, in, n, d_out)
#define CALL(R)                                   \
  do {                                            \
    if (dtype == ZC_F32) LAUNCH(R, kF32);         \
    else if (dtype == ZC_BF16) LAUNCH(R, kBF16);  \
    else LAUNCH(R, kF16);                         \
  } while (0)
  ZC_DISPATCH_RATE(rate, CALL)
#undef CALL
#undef LAUNCH
  return finish_launch();
}

int zc_compress(const float* d_in, size_t n, int rate, void* d_out, size_t out_cap, void* stream) {
  return launch_compress(d_in, ZC_F32, n, rate, d_out, out_cap, stream);
}

int zc_decompress(const void* d_in, size_t n, int rate, float* d_out, void* stream) {
  return launch_decompress(d_in, n, rate, ZC_F32, d_out, stream);
}

int zc_compress_half(const void* d_in, int dtype, size_t n, int rate, void* d_out, size_t out_cap, void* stream) {
  if (dtype != ZC_BF16 && dtype != ZC_F16) return ZC_ERR_DTYPE;
  return launch_compress(d_in, dtype, n, rate, d_out, out_cap, stream);
}

int zc_decompress_half(const void* d_in, size_t n, int rate, int dtype, void* d_out, void* stream) {
  if (dtype != ZC_BF16 && dtype != ZC_F16) return ZC_ERR_DTYPE;
  return launch_decompress(d_in, n, rate, dtype, d_out, stream);
}

static int launch_reduce(const void* const* d_in, int k, const float* d_local, size_t n, int rate, void* d_out,
                         size_t out_cap, float* d_out_raw, void* stream) {
  const bool raw_out = d_out_raw != nullptr;
  if (!zc_rate_supported(rate)) return ZC_ERR_RATE;
  if (k < 1 || k > kMaxChunks) return ZC_ERR_K;
  if (n == 0) return ZC_OK;
  if (!d_in || (!raw_out && !d_out)) return ZC_ERR_NULL;
  ChunkPointers chunks;
  for (int c = 0; c < kMaxChunks; ++c) chunks.p[c] = nullptr;
  for (int c = 0; c < k; ++c) {
    if (!d_in[c]) return ZC_ERR_NULL;
    if (!aligned16(d_in[c])) return ZC_ERR_ALIGN;
    chunks.p[c] = static_cast<const uint8_t*>(d_in[c]);
  }
  if (!aligned16(d_out) || !aligned16(d_out_raw) || !aligned16(d_local)) return ZC_ERR_ALIGN;
  if (n > kMaxValues) return ZC_ERR_SIZE;
  if (!raw_out && out_cap < zc_compressed_size(n, rate)) return ZC_ERR_CAPACITY;
  hipStream_t s = static_cast<hipStream_t>(stream);
  uint8_t* out = static_cast<uint8_t*>(d_out);
#define LAUNCH_K(R, LOCAL, RAW, K)                                                                            \
  hipLaunchKernelGGL((reduce_kernel<R, reduce_unroll<R>(), LOCAL, RAW, K>), dim3(grid_for(n, RAW ? kReduceRaw : kReduce, R, reduce_unroll<R>())),    \
                     dim3(kThreads), 0, s, chunks, k, d_local, n, out, d_out_raw)
#define LAUNCH(R, LOCAL, RAW)                 \
  do {                                        \
    if (k == 2) LAUNCH_K(R, LOCAL, RAW, 2);   \
    else LAUNCH_K(R, LOCAL, RAW, 0);          \
  } while (0)
#define CALL(R)                                   \
  do {                                            \
    if (d_local && raw_out) LAUNCH(R, true, true);        \
    else if (d_local) LAUNCH(R, true, false);     \
    else if (raw_out) LAUNCH(R, false, true);     \
    else LAUNCH(R, false, false);                 \
  } while (0)
  ZC_DISPATCH_RATE(rate, CALL)
#undef CALL
#undef LAUNCH
#undef LAUNCH_K
  return finish_launch();
}

int zc_reduce_compressed(const void* const* d_in, int k, size_t n, int rate, void* d_out, size_t out_cap,
                         void* stream) {
  return launch_reduce(d_in, k, nullptr, n, rate, d_out, out_cap, nullptr, stream);
}

int zc_reduce_mixed(const void* const* d_in, int k, const float* d_local, size_t n, int rate, void* d_out,
                    size_t out_cap, void* stream) {
  return launch_reduce(d_in, k, d_local, n, rate, d_out, out_cap, nullptr, stream);
}

int zc_reduce_decompress(const void* const* d_in, int k, const float* d_local, size_t n, int rate, float* d_out,
                         void* stream) {
  if (zc_rate_supported(rate) && k >= 1 && k <= kMaxChunks && n != 0 && !d_out) return ZC_ERR_NULL;
  return launch_reduce(d_in, k, d_local, n, rate, nullptr, 0, d_out, stream);
}

}  // extern "C"
