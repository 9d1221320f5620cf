// zc2d_kernels.hip -- gfx950 kernels and C ABI for the 4 x 4 block codec (see include/zc.h).
//
// One lane per block of 4 x 4 values, blocks taken in row-major block order with a grid
// stride, so that the 64 lanes of a wavefront read four contiguous 1 KiB spans (one per
// matrix row of the block row) and write one contiguous span of 64 * 2*RATE stream bytes.
// A block lives in registers from load to store; LDS holds only the coder's look-up table
// (1 KiB for the encoder, 22 KiB for the decoder).  No matrix cores: nothing here is a
// contraction.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include "../../include/zc.h"
#include "zc2d_codec.h"
#include "zc_half.h"

namespace {

constexpr int kThreads = 256;

__device__ __align__(16) const zc2d::ExpandTable g_expand = zc2d::build_expand_table();
__device__ __align__(16) const zc2d::TokenTable g_token = zc2d::build_token_table();

// Copy a table of WORDS 32-bit words to LDS, 16 bytes per lane and step: a lane issues all of
// its loads back to back and then writes (one wait for the whole table, not one per step).
// In a last, partial step of several the lanes beyond the table's end copy its first entry
// once more.
template <int WORDS>
__device__ __forceinline__ void stage_table(const uint32_t* __restrict__ src, uint32_t* dst) {
  static_assert(WORDS % 4 == 0, "table size");
  constexpr int kVecs = WORDS / 4;
  constexpr int kSteps = (kVecs + kThreads - 1) / kThreads;
  if constexpr (kSteps == 1) {
    if (threadIdx.x < kVecs) reinterpret_cast<uint4*>(dst)[threadIdx.x] = reinterpret_cast<const uint4*>(src)[threadIdx.x];
  } else {
    uint4 v[kSteps];
    int idx[kSteps];
#pragma unroll
    for (int i = 0; i < kSteps; ++i) {
      idx[i] = threadIdx.x + i * kThreads;
      if ((i + 1) * kThreads > kVecs && idx[i] >= kVecs) idx[i] = 0;
      v[i] = reinterpret_cast<const uint4*>(src)[idx[i]];
    }
#pragma unroll
    for (int i = 0; i < kSteps; ++i) reinterpret_cast<uint4*>(dst)[idx[i]] = v[i];
    __builtin_amdgcn_sched_group_barrier(0x020, kSteps, 0);   // (for the instruction scheduler: the loads first,
    __builtin_amdgcn_sched_group_barrier(0x200, kSteps, 0);   // then the LDS writes)
  }
  __syncthreads();
}
// Workgroups per CU in the grid (measured: the decoder-bound kernels like a few more than
// the compress kernel).  Only a build with -DZC_TUNING_KNOBS lets ZC2D_WORKGROUPS_PER_CU override both; the shipped library reads no environment variable.
constexpr int kCompressWorkgroupsPerCU = 16, kDecodeWorkgroupsPerCU = 48;

// The wavefront-wide votes of the codec: lanes(p) is the set of lanes where p holds (one
// comparison each, so that the compare instruction's own mask is the set), some(set) whether
// it is non-empty; any_lane_active(p) = some(lanes(p)).
struct AnyLane {
  __device__ uint64_t lanes(bool p) const { return __builtin_amdgcn_ballot_w64(p); }
  __device__ bool some(uint64_t set) const { return set != 0; }
  __device__ bool operator()(bool p) const { return __builtin_amdgcn_ballot_w64(p) != 0; }
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Shape of the matrix and of the walk over its blocks; the same for every lane.
struct Walk {
  size_t rows, cols;
  size_t bc, blocks;        // blocks per block row, blocks in all
  size_t stride;            // lanes in the grid: a lane's next block is `stride` blocks on
  size_t step_bi, step_bj;  // stride / bc, stride % bc
};

// A lane's place in the walk.  Advancing costs additions only: no division per block.
struct Cursor {
  size_t b, bi, bj;   // block index, block row, block column
  size_t first;       // index of the block's first value, (4 * bi) * cols + 4 * bj

  __device__ __forceinline__ void start(const Walk& w, size_t b0) {
    b = b0;
    bi = b0 / w.bc;
    bj = b0 - bi * w.bc;
    first = 4 * bi * w.cols + 4 * bj;
  }
  __device__ __forceinline__ void advance(const Walk& w) {
    b += w.stride;
    bi += w.step_bi;
    bj += w.step_bj;
    first += 4 * (w.step_bi * w.cols + w.step_bj);
    if (bj >= w.bc) {
      bj -= w.bc;
      bi += 1;
      first += 4 * w.cols - 4 * w.bc;
    }
  }
  // all 16 values inside the matrix and every row of the block 16-byte aligned
  __device__ __forceinline__ bool whole(const Walk& w) const { return (w.cols & 3) == 0 && 4 * bi + 4 <= w.rows; }
};

// The block under the cursor as fp32 bit patterns; parts that stick out of the matrix
// repeat the last valid row / column.  DT: the matrix holds fp32, or bf16 / fp16 values
// that are widened (exactly) on the way in.
template <int DT>
__device__ __forceinline__ void load_block(const void* in, const Walk& w, const Cursor& c, uint32_t (&x)[16]) {
  if (c.whole(w)) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      if constexpr (DT == kF32) {
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(static_cast<const float*>(in) + c.first + r * w.cols));
        x[4 * r] = v.x; x[4 * r + 1] = v.y; x[4 * r + 2] = v.z; x[4 * r + 3] = v.w;
      } else {
        const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(static_cast<const uint16_t*>(in) + c.first + r * w.cols));
        x[4 * r] = widen_half<DT>(v.x & 0xFFFFu); x[4 * r + 1] = widen_half<DT>(v.x >> 16);
        x[4 * r + 2] = widen_half<DT>(v.y & 0xFFFFu); x[4 * r + 3] = widen_half<DT>(v.y >> 16);
      }
    }
  } else {
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        size_t rr = 4 * c.bi + r, cc = 4 * c.bj + q;
        rr = rr < w.rows ? rr : w.rows - 1;
        cc = cc < w.cols ? cc : w.cols - 1;
        if constexpr (DT == kF32) x[4 * r + q] = static_cast<const uint32_t*>(in)[rr * w.cols + cc];
        else x[4 * r + q] = widen_half<DT>(static_cast<const uint16_t*>(in)[rr * w.cols + cc]);
      }
  }
}

// The reverse; half-precision values are rounded to nearest, ties to even.
template <int DT>
__device__ __forceinline__ void store_block(void* out, const Walk& w, const Cursor& c, const float (&y)[16]) {
  if (c.whole(w)) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      if constexpr (DT == kF32) {
        const u32x4 v = {__float_as_uint(y[4 * r]), __float_as_uint(y[4 * r + 1]), __float_as_uint(y[4 * r + 2]),
                         __float_as_uint(y[4 * r + 3])};
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(static_cast<float*>(out) + c.first + r * w.cols));
      } else {
        const u32x2 v = {narrow_half<DT>(y[4 * r]) | narrow_half<DT>(y[4 * r + 1]) << 16,
                         narrow_half<DT>(y[4 * r + 2]) | narrow_half<DT>(y[4 * r + 3]) << 16};
        __builtin_nontemporal_store(v, reinterpret_cast<u32x2*>(static_cast<uint16_t*>(out) + c.first + r * w.cols));
      }
    }
  } else {
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const size_t rr = 4 * c.bi + r, cc = 4 * c.bj + q;
        if (rr < w.rows && cc < w.cols) {
          if constexpr (DT == kF32) static_cast<float*>(out)[rr * w.cols + cc] = y[4 * r + q];
          else static_cast<uint16_t*>(out)[rr * w.cols + cc] = (uint16_t)narrow_half<DT>(y[4 * r + q]);
        }
      }
  }
}

template <int NW>
__device__ __forceinline__ void load_words(const uint8_t* p, uint32_t (&W)[NW]) {
  if constexpr (NW == 1) {
    W[0] = *reinterpret_cast<const uint32_t*>(p);
  } else if constexpr (NW == 2) {
    const u32x2 v = *reinterpret_cast<const u32x2*>(p);
    W[0] = v.x; W[1] = v.y;
  } else {
#pragma unroll
    for (int i = 0; i < NW / 4; ++i) {
      const u32x4 v = reinterpret_cast<const u32x4*>(p)[i];
      W[4 * i] = v.x; W[4 * i + 1] = v.y; W[4 * i + 2] = v.z; W[4 * i + 3] = v.w;
    }
  }
}

template <int NW>
__device__ __forceinline__ void store_words(uint8_t* p, const uint32_t (&W)[NW]) {
  if constexpr (NW == 1) {
    *reinterpret_cast<uint32_t*>(p) = W[0];
  } else if constexpr (NW == 2) {
    const u32x2 v = {W[0], W[1]};
    *reinterpret_cast<u32x2*>(p) = v;
  } else {
#pragma unroll
    for (int i = 0; i < NW / 4; ++i) {
      const u32x4 v = {W[4 * i], W[4 * i + 1], W[4 * i + 2], W[4 * i + 3]};
      reinterpret_cast<u32x4*>(p)[i] = v;
    }
  }
}

template <int RATE, int DT>
__global__ __launch_bounds__(kThreads) void compress2d_kernel(const void* __restrict__ in, Walk w,
                                                              uint8_t* __restrict__ out) {
  __shared__ __attribute__((aligned(16))) uint32_t expand[256];
  stage_table<256>(g_expand.v, expand);
  constexpr int NW = zc2d::Traits<RATE>::kWords;
  const size_t b0 = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (b0 >= w.blocks) return;
  Cursor cur;
  cur.start(w, b0);
  uint32_t x[16];
  load_block<DT>(in, w, cur, x);
  // The first block has to have arrived before the loop starts: with loads still in flight
  // at its entry, every pass would wait for its own prefetch as well (loads return in order).
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
  for (;;) {
    // The loads of the lane's next block, if it has one, are issued before its current
    // block is coded.
    Cursor next = cur;
    next.advance(w);
    const bool more = next.b < w.blocks;
    uint32_t xn[16], W[NW];
    if (more) load_block<DT>(in, w, next, xn);
    zc2d::encode_block<RATE>(x, expand, W, AnyLane());
    store_words<NW>(out + cur.b * zc2d::Traits<RATE>::kBlockBytes, W);
    if (!more) break;
#pragma unroll
    for (int i = 0; i < 16; ++i) x[i] = xn[i];
    cur = next;
  }
}

template <int RATE, int DT>
__global__ __launch_bounds__(kThreads) void decompress2d_kernel(const uint8_t* __restrict__ in, Walk w,
                                                                void* __restrict__ out) {
  __shared__ __attribute__((aligned(16))) uint32_t token[zc2d::kTokenRows << zc2d::kLookahead];
  stage_table<(zc2d::kTokenRows << zc2d::kLookahead)>(g_token.v, token);
  constexpr int NW = zc2d::Traits<RATE>::kWords;
  const size_t b0 = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (b0 >= w.blocks) return;
  Cursor cur;
  cur.start(w, b0);
  uint32_t W[NW];
  load_words<NW>(in + cur.b * zc2d::Traits<RATE>::kBlockBytes, W);
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0), for the same reason as in the compress kernel
  for (;;) {
    Cursor next = cur;
    next.advance(w);
    const bool more = next.b < w.blocks;
    uint32_t Wn[NW];
    if (more) load_words<NW>(in + next.b * zc2d::Traits<RATE>::kBlockBytes, Wn);   // the next block's stream, ahead of time
    float y[16];
    zc2d::decode_block<RATE>(W, token, y, AnyLane());
    store_block<DT>(out, w, cur, y);
    if (!more) break;
#pragma unroll
    for (int i = 0; i < NW; ++i) W[i] = Wn[i];
    cur = next;
  }
}

struct ChunkPointers2d {
  const uint8_t* p[16];
};

// The reduce-scatter step on matrix-shaped messages: block b of the k chunks is decoded,
// the 16 values are added in registers in chunk order, and the sum is encoded; where the
// block sticks out of the matrix its fill is taken from the sum's last valid row / column.
// LOCAL: a raw fp32 matrix is added last (a ring hop's own contribution); RAW_OUT: the sum
// is stored as an fp32 matrix instead of being encoded (the last hop).
// (The plain form at the low rates is two registers away from a sixth wavefront per SIMD, which
// it gains from: the compiler is told to stay within that; the other forms would spill.)
template <int RATE, bool LOCAL, bool RAW_OUT>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(RATE <= 4 && !LOCAL && !RAW_OUT ? 6 : 1)))
void reduce2d_kernel(ChunkPointers2d chunks, int k, const float* local, Walk w, uint8_t* out, float* out_raw) {
  __shared__ __attribute__((aligned(16))) uint32_t expand[256];
  __shared__ __attribute__((aligned(16))) uint32_t token[zc2d::kTokenRows << zc2d::kLookahead];
  for (int i = threadIdx.x; i < 256 / 4; i += kThreads)
    reinterpret_cast<uint4*>(expand)[i] = reinterpret_cast<const uint4*>(g_expand.v)[i];
  stage_table<(zc2d::kTokenRows << zc2d::kLookahead)>(g_token.v, token);   // (its barrier covers both tables)
  constexpr int NW = zc2d::Traits<RATE>::kWords;
  const size_t b0 = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (b0 >= w.blocks) return;
  Cursor cur;
  cur.start(w, b0);
  for (;;) {
    const size_t at = cur.b * zc2d::Traits<RATE>::kBlockBytes;
    float sum[16];
    {
      uint32_t W[NW];
      load_words<NW>(chunks.p[0] + at, W);
      zc2d::decode_block<RATE>(W, token, sum, AnyLane());
    }
#pragma unroll 1
    for (int j = 1; j < k; ++j) {
      uint32_t W[NW];
      int32_t q[16];
      load_words<NW>(chunks.p[j] + at, W);
      const uint32_t E = zc2d::decode_block_fixed<RATE>(W, token, q, AnyLane());
      // scale and add in one fused step, unless some lane's exponent byte is one where the
      // scaling may round or overflow (tiny or huge blocks, arbitrary bytes)
      if (AnyLane()(!zc2d::scaling_is_exact(E))) {
        float y[16];
        zc2d::scale_block(q, E, y);
#pragma unroll
        for (int i = 0; i < 16; ++i) sum[i] += y[i];
      } else {
        zc2d::accumulate_scaled(q, E, sum);
      }
    }
    if constexpr (LOCAL) {
      // (where the block sticks out of the matrix the clamped loads add copies of edge values;
      // those positions are refilled from the sum or dropped below)
      uint32_t mine[16];
      load_block<kF32>(local, w, cur, mine);
#pragma unroll
      for (int i = 0; i < 16; ++i) sum[i] += __uint_as_float(mine[i]);
    }
    if constexpr (RAW_OUT) {
      store_block<kF32>(out_raw, w, cur, sum);
      cur.advance(w);
      if (cur.b >= w.blocks) break;
      continue;
    }
    uint32_t x[16];
    if (cur.whole(w) || (4 * cur.bi + 4 <= w.rows && 4 * cur.bj + 4 <= w.cols)) {
#pragma unroll
      for (int i = 0; i < 16; ++i) x[i] = __float_as_uint(sum[i]);
    } else {
      const uint32_t rv = (uint32_t)(w.rows - 4 * cur.bi < 4 ? w.rows - 4 * cur.bi : 4);
      const uint32_t cv = (uint32_t)(w.cols - 4 * cur.bj < 4 ? w.cols - 4 * cur.bj : 4);
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          // value at (min(r, rv-1), min(q, cv-1)), picked without indexing registers by a variable
          float v = sum[0];
#pragma unroll
          for (int rr = 0; rr < 4; ++rr)
#pragma unroll
            for (int qq = 0; qq < 4; ++qq) {
              const bool pick = (uint32_t)rr == ((uint32_t)r < rv ? (uint32_t)r : rv - 1) &&
                                (uint32_t)qq == ((uint32_t)q < cv ? (uint32_t)q : cv - 1);
              v = pick ? sum[4 * rr + qq] : v;
            }
          x[4 * r + q] = __float_as_uint(v);
        }
    }
    uint32_t W[NW];
    zc2d::encode_block<RATE>(x, expand, W, AnyLane());
    store_words<NW>(out + at, W);
    cur.advance(w);
    if (cur.b >= w.blocks) break;
  }
}

int compute_units() {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 256;
  return cus;
}

int workgroups_per_cu(int preset) {
#ifdef ZC_TUNING_KNOBS
  if (const char* e = getenv("ZC2D_WORKGROUPS_PER_CU")) {
    const int v = atoi(e);
    if (v >= 1 && v <= 4096) return v;
  }
#endif
  return preset;
}

unsigned grid_for(size_t blocks, int preset) {
  const size_t groups = (blocks + kThreads - 1) / kThreads;
  const size_t cap = (size_t)compute_units() * (size_t)workgroups_per_cu(preset);
  return (unsigned)(groups < cap ? groups : cap);
}

Walk walk_for(size_t rows, size_t cols, unsigned grid) {
  Walk w;
  w.rows = rows;
  w.cols = cols;
  w.bc = (cols + 3) / 4;
  w.blocks = ((rows + 3) / 4) * w.bc;
  w.stride = (size_t)grid * kThreads;
  w.step_bi = w.stride / w.bc;
  w.step_bj = w.stride % w.bc;
  return w;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
constexpr size_t kMaxValues = (size_t)1 << 40;

}  // namespace

#define ZC2D_DISPATCH_RATE(rate, CALL) \
  switch (rate) {                      \
    case 2: CALL(2); break;            \
    case 4: CALL(4); break;            \
    case 8: CALL(8); break;            \
    case 16: CALL(16); break;          \
    default: return ZC_ERR_RATE;       \
  }

namespace {

template <int DT>
int launch_compress2d(const void* d_in, size_t rows, size_t cols, int rate, void* d_out, size_t out_cap, void* stream) {
  if (!zc2d_rate_supported(rate)) return ZC_ERR_RATE;
  if (rows == 0 || cols == 0) return ZC_OK;
  if (!d_in || !d_out) return ZC_ERR_NULL;
  if (!aligned16(d_in) || !aligned16(d_out)) return ZC_ERR_ALIGN;
  if (rows > kMaxValues || cols > kMaxValues || rows > kMaxValues / cols) return ZC_ERR_SIZE;
  if (out_cap < zc2d_compressed_size(rows, cols, rate)) return ZC_ERR_CAPACITY;
  const size_t blocks = ((rows + 3) / 4) * ((cols + 3) / 4);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const unsigned grid = grid_for(blocks, kCompressWorkgroupsPerCU);
  const Walk w = walk_for(rows, cols, grid);
#define CALL(R) hipLaunchKernelGGL((compress2d_kernel<R, DT>), dim3(grid), dim3(kThreads), 0, s, d_in, w, static_cast<uint8_t*>(d_out))
  ZC2D_DISPATCH_RATE(rate, CALL)
#undef CALL
  return hipGetLastError() == hipSuccess ? ZC_OK : ZC_ERR_LAUNCH;
}

template <int DT>
int launch_decompress2d(const void* d_in, size_t rows, size_t cols, int rate, void* d_out, void* stream) {
  if (!zc2d_rate_supported(rate)) return ZC_ERR_RATE;
  if (rows == 0 || cols == 0) return ZC_OK;
  if (!d_in || !d_out) return ZC_ERR_NULL;
  if (!aligned16(d_in) || !aligned16(d_out)) return ZC_ERR_ALIGN;
  if (rows > kMaxValues || cols > kMaxValues || rows > kMaxValues / cols) return ZC_ERR_SIZE;
  const size_t blocks = ((rows + 3) / 4) * ((cols + 3) / 4);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const unsigned grid = grid_for(blocks, kDecodeWorkgroupsPerCU);
  const Walk w = walk_for(rows, cols, grid);
#define CALL(R) hipLaunchKernelGGL((decompress2d_kernel<R, DT>), dim3(grid), dim3(kThreads), 0, s, static_cast<const uint8_t*>(d_in), w, d_out)
  ZC2D_DISPATCH_RATE(rate, CALL)
#undef CALL
  return hipGetLastError() == hipSuccess ? ZC_OK : ZC_ERR_LAUNCH;
}

int launch_reduce2d(const void* const* d_in, int k, const float* d_local, size_t rows, size_t cols, int rate, void* d_out,
                    size_t out_cap, float* d_out_raw, void* stream) {
  const bool raw_out = d_out_raw != nullptr;
  if (!zc2d_rate_supported(rate)) return ZC_ERR_RATE;
  if (k < 1 || k > 16) return ZC_ERR_K;
  if (rows == 0 || cols == 0) return ZC_OK;
  if (!d_in || (!raw_out && !d_out)) return ZC_ERR_NULL;
  ChunkPointers2d chunks;
  for (int j = 0; j < 16; ++j) chunks.p[j] = nullptr;
  for (int j = 0; j < k; ++j) {
    if (!d_in[j]) return ZC_ERR_NULL;
    if (!aligned16(d_in[j])) return ZC_ERR_ALIGN;
    chunks.p[j] = static_cast<const uint8_t*>(d_in[j]);
  }
  if (!aligned16(d_out) || !aligned16(d_out_raw) || !aligned16(d_local)) return ZC_ERR_ALIGN;
  if (rows > kMaxValues || cols > kMaxValues || rows > kMaxValues / cols) return ZC_ERR_SIZE;
  if (!raw_out && out_cap < zc2d_compressed_size(rows, cols, rate)) return ZC_ERR_CAPACITY;
  const size_t blocks = ((rows + 3) / 4) * ((cols + 3) / 4);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const unsigned grid = grid_for(blocks, kDecodeWorkgroupsPerCU);
  const Walk w = walk_for(rows, cols, grid);
  uint8_t* out = static_cast<uint8_t*>(d_out);
#define LAUNCH(R, LOCAL, RAW) \
  hipLaunchKernelGGL((reduce2d_kernel<R, LOCAL, RAW>), dim3(grid), dim3(kThreads), 0, s, chunks, k, d_local, w, out, d_out_raw)
#define CALL(R)                                    \
  do {                                             \
    if (d_local && raw_out) LAUNCH(R, true, true); \
    else if (d_local) LAUNCH(R, true, false);      \
    else if (raw_out) LAUNCH(R, false, true);      \
    else LAUNCH(R, false, false);                  \
  } while (0)
  ZC2D_DISPATCH_RATE(rate, CALL)
#undef CALL
#undef LAUNCH
  return hipGetLastError() == hipSuccess ? ZC_OK : ZC_ERR_LAUNCH;
}

}  // namespace

extern "C" {

int zc2d_rate_supported(int rate) { return rate == 2 || rate == 4 || rate == 8 || rate == 16; }

size_t zc2d_compressed_size(size_t rows, size_t cols, int rate) {
  if (!zc2d_rate_supported(rate)) return 0;
  return ((rows + 3) / 4) * ((cols + 3) / 4) * (size_t)(2 * rate);
}

int zc2d_compress(const float* d_in, size_t rows, size_t cols, int rate, void* d_out, size_t out_cap, void* stream) {
  return launch_compress2d<kF32>(d_in, rows, cols, rate, d_out, out_cap, stream);
}

int zc2d_decompress(const void* d_in, size_t rows, size_t cols, int rate, float* d_out, void* stream) {
  return launch_decompress2d<kF32>(d_in, rows, cols, rate, d_out, stream);
}

int zc2d_compress_half(const void* d_in, int dtype, size_t rows, size_t cols, int rate, void* d_out, size_t out_cap,
                       void* stream) {
  if (dtype == ZC_BF16) return launch_compress2d<kBF16>(d_in, rows, cols, rate, d_out, out_cap, stream);
  if (dtype == ZC_F16) return launch_compress2d<kF16>(d_in, rows, cols, rate, d_out, out_cap, stream);
  return ZC_ERR_DTYPE;
}

int zc2d_decompress_half(const void* d_in, size_t rows, size_t cols, int rate, int dtype, void* d_out, void* stream) {
  if (dtype == ZC_BF16) return launch_decompress2d<kBF16>(d_in, rows, cols, rate, d_out, stream);
  if (dtype == ZC_F16) return launch_decompress2d<kF16>(d_in, rows, cols, rate, d_out, stream);
  return ZC_ERR_DTYPE;
}

int zc2d_reduce_compressed(const void* const* d_in, int k, size_t rows, size_t cols, int rate, void* d_out,
                           size_t out_cap, void* stream) {
  return launch_reduce2d(d_in, k, nullptr, rows, cols, rate, d_out, out_cap, nullptr, stream);
}

int zc2d_reduce_mixed(const void* const* d_in, int k, const float* d_local, size_t rows, size_t cols, int rate, void* d_out,
                      size_t out_cap, void* stream) {
  return launch_reduce2d(d_in, k, d_local, rows, cols, rate, d_out, out_cap, nullptr, stream);
}

int zc2d_reduce_decompress(const void* const* d_in, int k, const float* d_local, size_t rows, size_t cols, int rate,
                           float* d_out, void* stream) {
  if (zc2d_rate_supported(rate) && k >= 1 && k <= 16 && rows != 0 && cols != 0 && !d_out) return ZC_ERR_NULL;
  return launch_reduce2d(d_in, k, d_local, rows, cols, rate, nullptr, 0, d_out, stream);
}

}  // extern "C"
