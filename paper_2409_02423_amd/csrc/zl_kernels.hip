// zl_kernels.hip -- gfx950 kernels and C ABI for the lossless codec (see include/zc.h).
//
// One workgroup of 256 lanes per chunk of 8192 words; a lane owns one group of 32 words
// (its eight 16-byte reads), so residuals, the bit transpose and the test for empty
// planes all stay in registers.  The non-zero planes are compacted through LDS (a
// workgroup-wide prefix sum of the per-lane counts gives every lane its place) and
// leave as one contiguous span per chunk.
//
// Chunks have data-dependent sizes, so a chunk's place in the stream is the sum of the
// sizes before it.  That sum is formed in the same launch: chunk numbers are handed out
// by a counter in the order in which workgroups start, a workgroup publishes its own
// size in the stream's table as soon as it knows it, then adds up its predecessors'
// entries, 64 at a time, back to the nearest one that already holds a running total,
// and replaces its entry by its own running total.  Every entry a workgroup waits for
// belongs to a workgroup that has started and that publishes before it waits, so every
// wait ends; a spin limit turns the impossible case into an error mark in the header.
// The table is part of the stream (the decoder needs it) and the counter ends up as the
// header's chunk count: no memory beyond input and output is used.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/zc.h"
#include "zl_codec.h"

namespace {

constexpr int kThreads = zl::kGroups;
constexpr uint32_t kSpinLimit = 1u << 22;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct Header {
  uint32_t magic;
  uint32_t chunks;   // while compressing: chunk numbers handed out so far
  uint64_t n;
  uint64_t total;
  uint64_t flaw;     // zero in a valid stream
};
static_assert(sizeof(Header) == zl::kHeaderBytes, "header layout");

__global__ __launch_bounds__(256) void zero_words_kernel(uint64_t* p, size_t count) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (size_t)gridDim.x * 256) p[i] = 0;
}

// The stream of an empty message: the header alone.
__global__ void empty_stream_kernel(Header* header) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    header->magic = zl::kMagic;
    header->chunks = 0;
    header->n = 0;
    header->total = zl::kHeaderBytes;
    header->flaw = 0;
  }
}

// Inclusive prefix sum over the wavefront.
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t v, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t up = (uint32_t)__shfl_up((int)v, d);
    v += lane >= d ? up : 0u;
  }
  return v;
}

__device__ __forceinline__ uint64_t wave_sum64(uint64_t v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    const uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)v, d);
    const uint32_t hi = (uint32_t)__shfl_xor((int)(uint32_t)(v >> 32), d);
    v += (uint64_t)hi << 32 | lo;
  }
  return v;
}

// Exclusive prefix sum of `count` over the 256 lanes of the workgroup; `total` gets the sum.
__device__ __forceinline__ uint32_t workgroup_exclusive_sum(uint32_t count, uint32_t* wave_totals, uint32_t& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t incl = wave_inclusive_sum(count, lane);
  if (lane == 63) wave_totals[wave] = incl;
  __syncthreads();
  uint32_t before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < kThreads / 64; ++w) {
    const uint32_t t = wave_totals[w];
    before += w < wave ? t : 0u;
    all += t;
  }
  total = all;
  return before + incl - count;
}

// Sum of the sizes of chunks 0..c-1, read from the table (run by one whole wavefront).
// Returns false if an entry stayed empty for kSpinLimit polls.
__device__ bool bytes_before(uint64_t* table, uint32_t c, int lane, uint64_t& before) {
  uint64_t sum = 0;
  int64_t base = (int64_t)c - 1;
  while (base >= 0) {
    const int64_t idx = base - lane;
    uint64_t s = 0;
    uint32_t first = 64;
    uint32_t polls = 0;
    for (;;) {
      s = idx >= 0 ? __hip_atomic_load(&table[idx], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : zl::kEnd;
      const uint64_t totals = __builtin_amdgcn_ballot_w64((s >> 62) == 2u);
      const uint64_t empty = __builtin_amdgcn_ballot_w64((s >> 62) == 0u);
      first = totals ? (uint32_t)__builtin_ctzll(totals) : 64u;
      const uint64_t needed = first >= 63u ? ~0ull : ((2ull << first) - 1ull);
      if ((empty & needed) == 0) break;
      if (++polls > kSpinLimit) return false;
      __builtin_amdgcn_s_sleep(2);
    }
    sum += wave_sum64((uint32_t)lane <= first ? (s & zl::kValueMask) : 0ull);
    if (first != 64u) break;
    base -= 64;
  }
  before = sum;
  return true;
}

__global__ __launch_bounds__(kThreads) void zl_compress_kernel(const uint32_t* __restrict__ in, size_t n, uint8_t* out,
                                                               uint32_t chunks) {
  __shared__ uint32_t stage[zl::kChunkWords];
  __shared__ uint32_t wave_totals[kThreads / 64];
  __shared__ uint32_t my_chunk;
  __shared__ uint64_t my_start;
  __shared__ uint32_t failed;
  Header* header = reinterpret_cast<Header*>(out);
  uint64_t* table = reinterpret_cast<uint64_t*>(out + zl::kHeaderBytes);
  uint8_t* payload = out + zl::kHeaderBytes + 8 * (size_t)chunks;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  if (tid == 0) {
    my_chunk = __hip_atomic_fetch_add(&header->chunks, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    failed = 0;
  }
  __syncthreads();
  const uint32_t c = my_chunk;
  if (c >= chunks) return;   // cannot happen with one workgroup per chunk; keeps every access in bounds regardless

  // the lane's group: words 1024*t + 4*tid .. +3 of the chunk, t = 0..7
  const size_t base = (size_t)c * zl::kChunkWords;
  uint32_t w[32];
  if (base + zl::kChunkWords <= n) {
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(in + base + 1024 * t + 4 * tid));
      w[4 * t] = v.x; w[4 * t + 1] = v.y; w[4 * t + 2] = v.z; w[4 * t + 3] = v.w;
    }
  } else {
#pragma unroll
    for (int j = 0; j < 32; ++j) {
      const size_t i = base + 1024 * (j >> 2) + 4 * tid + (j & 3);
      w[j] = i < n ? in[i] : 0u;
    }
  }
  uint32_t reference;
  const uint32_t bitmap = zl::to_planes(w, reference);
  const uint32_t count = (uint32_t)__builtin_popcount(bitmap);
  uint32_t total_words;
  uint32_t pos = workgroup_exclusive_sum(count, wave_totals, total_words);
#pragma unroll
  for (int k = 0; k < 32; ++k)
    if ((bitmap >> k) & 1u) stage[pos++] = w[k];
  const uint64_t bytes = zl::kFixedChunkBytes + 4ull * total_words;

  if (wave == 0) {
    if (lane == 0)
      __hip_atomic_store(&table[c], (c == 0 ? zl::kEnd : zl::kOwnSize) | bytes, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    uint64_t before = 0;
    const bool ok = c == 0 || bytes_before(table, c, lane, before);
    if (lane == 0) {
      if (!ok) {
        failed = 1;
        __hip_atomic_fetch_or(&header->flaw, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      // publish a running total in any case, so that no later chunk waits for this one
      if (c != 0)
        __hip_atomic_store(&table[c], zl::kEnd | (before + bytes), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      my_start = before;
      if (c == chunks - 1 && ok) {   // the last chunk completes the header
        __hip_atomic_store(&header->magic, zl::kMagic, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&header->n, (uint64_t)n, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&header->total, zl::kHeaderBytes + 8ull * chunks + before + bytes, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
  __syncthreads();
  if (failed) return;   // the stream is marked flawed; nothing of this chunk is written

  uint32_t* dst = reinterpret_cast<uint32_t*>(payload + my_start);
  dst[tid] = reference;
  dst[kThreads + tid] = bitmap;
  dst += 2 * kThreads;
  for (uint32_t i = tid; i < total_words; i += kThreads) dst[i] = stage[i];
}

// in_bytes: size of the buffer that holds the stream; every read stays below it.
__global__ __launch_bounds__(kThreads) void zl_decompress_kernel(const uint8_t* __restrict__ in, size_t in_bytes, size_t n,
                                                                 uint32_t* __restrict__ out, uint32_t chunks) {
  __shared__ uint32_t stage[zl::kChunkWords + 64];   // a lane may look one past its last plane
  __shared__ uint32_t wave_totals[kThreads / 64];
  const uint64_t* table = reinterpret_cast<const uint64_t*>(in + zl::kHeaderBytes);
  const uint64_t room = in_bytes - zl::kHeaderBytes - 8 * (uint64_t)chunks;   // the host checked that this is not negative
  const uint32_t* payload = reinterpret_cast<const uint32_t*>(in + zl::kHeaderBytes + 8 * (size_t)chunks);
  const int tid = threadIdx.x;
  const uint32_t c = blockIdx.x;

  // the chunk's span, clamped to the buffer and to whole words
  uint64_t end = table[c] & zl::kValueMask, start = c ? table[c - 1] & zl::kValueMask : 0;
  end = end < room ? end : room;
  start = start < end ? start : end;
  const uint64_t first_word = (start + 3) / 4, words = end / 4 > first_word ? end / 4 - first_word : 0;
  const uint32_t* src = payload + first_word;

  const uint32_t reference = (uint64_t)tid < words ? src[tid] : 0u;
  const uint32_t bitmap = (uint64_t)(kThreads + tid) < words ? src[kThreads + tid] : 0u;
  uint32_t total_words;
  uint32_t pos = workgroup_exclusive_sum((uint32_t)__builtin_popcount(bitmap), wave_totals, total_words);
  const uint64_t stored = words > 2 * kThreads ? words - 2 * kThreads : 0;
  for (uint32_t i = tid; i < total_words; i += kThreads) stage[i] = i < stored ? src[2 * kThreads + i] : 0u;
  __syncthreads();

  uint32_t p[32];
#pragma unroll
  for (int k = 0; k < 32; ++k) {
    const bool present = (bitmap >> k) & 1u;
    p[k] = present ? stage[pos] : 0u;
    pos += present ? 1u : 0u;
  }
  zl::from_planes(p, reference);

  const size_t base = (size_t)c * zl::kChunkWords;
  if (base + zl::kChunkWords <= n) {
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const u32x4 v = {p[4 * t], p[4 * t + 1], p[4 * t + 2], p[4 * t + 3]};
      __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(out + base + 1024 * t + 4 * tid));
    }
  } else {
#pragma unroll
    for (int j = 0; j < 32; ++j) {
      const size_t i = base + 1024 * (j >> 2) + 4 * tid + (j & 3);
      if (i < n) out[i] = p[j];
    }
  }
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
constexpr size_t kMaxWords = (size_t)1 << 40;

size_t chunks_of(size_t n) { return (n + zl::kChunkWords - 1) / zl::kChunkWords; }

}  // namespace

extern "C" {

size_t zl_max_compressed_size(size_t n) {
  if (n > kMaxWords) return 0;
  return zl::kHeaderBytes + chunks_of(n) * (size_t)(8 + zl::kFixedChunkBytes + 4 * zl::kChunkWords);
}

int zl_compress(const void* d_in, size_t n, void* d_out, size_t out_cap, void* stream) {
  if (!d_out || (n && !d_in)) return ZC_ERR_NULL;
  if (!aligned16(d_in) || !aligned16(d_out)) return ZC_ERR_ALIGN;
  if (n > kMaxWords) return ZC_ERR_SIZE;
  if (out_cap < zl_max_compressed_size(n)) return ZC_ERR_CAPACITY;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t chunks = chunks_of(n);
  if (chunks == 0) {
    hipLaunchKernelGGL(empty_stream_kernel, dim3(1), dim3(64), 0, s, static_cast<Header*>(d_out));
    return hipGetLastError() == hipSuccess ? ZC_OK : ZC_ERR_LAUNCH;
  }
  // header and table start as zeros: the chunk counter, the empty table entries, the flaw mark
  // (a fill kernel rather than a memset node, so that the call can be captured in a graph)
  const size_t clear = (zl::kHeaderBytes + 8 * chunks) / 8;
  const unsigned zgrid = (unsigned)((clear + 255) / 256 < 1024 ? (clear + 255) / 256 : 1024);
  hipLaunchKernelGGL(zero_words_kernel, dim3(zgrid), dim3(256), 0, s, static_cast<uint64_t*>(d_out), clear);
  if (hipGetLastError() != hipSuccess) return ZC_ERR_LAUNCH;
  hipLaunchKernelGGL(zl_compress_kernel, dim3((unsigned)chunks), dim3(kThreads), 0, s, static_cast<const uint32_t*>(d_in), n,
                     static_cast<uint8_t*>(d_out), (uint32_t)chunks);
  return hipGetLastError() == hipSuccess ? ZC_OK : ZC_ERR_LAUNCH;
}

int zl_stream_bytes(const void* d_stream, size_t* h_bytes, void* stream) {
  if (!d_stream || !h_bytes) return ZC_ERR_NULL;
  Header h;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (hipMemcpyAsync(&h, d_stream, sizeof h, hipMemcpyDeviceToHost, s) != hipSuccess) return ZC_ERR_LAUNCH;
  if (hipStreamSynchronize(s) != hipSuccess) return ZC_ERR_LAUNCH;
  if (h.magic != zl::kMagic || h.flaw != 0) return ZC_ERR_STREAM;
  *h_bytes = (size_t)h.total;
  return ZC_OK;
}

int zl_decompress(const void* d_in, size_t in_bytes, size_t n, void* d_out, void* stream) {
  if (!d_in || (n && !d_out)) return ZC_ERR_NULL;
  if (!aligned16(d_in) || !aligned16(d_out)) return ZC_ERR_ALIGN;
  if (n > kMaxWords) return ZC_ERR_SIZE;
  const size_t chunks = chunks_of(n);
  if (in_bytes < zl::kHeaderBytes + 8 * chunks) return ZC_ERR_CAPACITY;
  if (chunks == 0) return ZC_OK;
  hipLaunchKernelGGL(zl_decompress_kernel, dim3((unsigned)chunks), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                     static_cast<const uint8_t*>(d_in), in_bytes, n, static_cast<uint32_t*>(d_out), (uint32_t)chunks);
  return hipGetLastError() == hipSuccess ? ZC_OK : ZC_ERR_LAUNCH;
}

}  // extern "C"
