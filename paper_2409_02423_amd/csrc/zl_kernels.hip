// zl_kernels.hip -- gfx950 kernels and C ABI for the lossless codec (see include/zc.h).
//
// One workgroup of 256 lanes per chunk of 8192 words; a lane owns one group of 32 words
// (its eight 16-byte reads), so residuals, the bit transpose and the test for empty
// planes all stay in registers.  A workgroup-wide prefix sum of the per-lane plane counts
// gives every lane its place in the chunk; each wavefront then moves its planes between
// registers and its contiguous span of the stream through 4 KiB of LDS of its own, half
// of its lanes at a time, with no further barrier (16 KiB of LDS per workgroup, so that
// seven workgroups fit on a CU and hide each other's waits).
//
// Chunks have data-dependent sizes, so a chunk's place in the stream is the sum of the
// sizes before it.  That sum is formed in the same launch.  The compress kernel runs about
// as many workgroups as fit on the chip at once; each takes chunk numbers from a counter,
// one after the other, and publishes a chunk's own size in the stream's table as soon as
// the chunk is coded.  The coded chunk then waits in registers while the workgroup codes
// its next one; only after that does the workgroup add up the entries of the chunks before
// the waiting one, 64 at a time, back to the nearest entry that already holds a running
// total, replace the chunk's entry by its own running total and write the chunk.  By then
// most of what the sum needs has arrived, so the look-back rarely has to poll.
// Every entry a workgroup waits for belongs to a chunk number taken by a running workgroup,
// and between taking a number and publishing that chunk's size a workgroup waits for no
// other workgroup; so every wait ends (also with several such kernels running at once,
// which a fixed assignment of chunks to workgroups would not survive).  A spin limit turns
// the impossible case into a flaw mark in the header.  The counter is the header's chunk
// count; it runs past its end (every workgroup asks once too often) and a last one-lane
// kernel sets it, and the rest of the header, to their final values.  The table is part
// of the stream (the decoder needs it): no memory beyond input and output is used.
// What bounds the kernel from below is the counter itself: 11.5 ns per request, however many
// workgroups ask (32768 requests alone take 0.38 ms); for 16-bit messages a workgroup of 512
// lanes therefore takes two chunks per request.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include "../../include/zc.h"
#include "zl_codec.h"

namespace {

constexpr int kThreads = zl::kGroups;
constexpr uint32_t kSpinLimit = 1u << 22;
// Chunks per workgroup of the compress kernel.  Two for 16-bit messages, whose compressor
// is otherwise bound by the chunk counter (half the bytes per chunk); one for 32-bit
// messages, where the wider workgroup's barriers cost more than the counter saves.
template <bool HALF> constexpr int chunks_per_workgroup() { return HALF ? 2 : 1; }
constexpr int kWaveStageWords = 32 * 33;   // planes of 32 lanes: a wavefront's LDS, one spare word per 32

// Where plane word i of a half-wavefront sits in its LDS.  Lanes reach their planes with a
// stride of their plane count (32 if nothing is dropped): the spare word per 32 keeps such
// strides off a single bank, and consecutive words stay consecutive for the copy.
__device__ __forceinline__ uint32_t staged(uint32_t i) { return i + (i >> 5); }

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

// Places of the planes within a chunk, from the per-lane counts.
struct Places {
  uint32_t in_wave;      // planes of lower lanes of the same wavefront
  uint32_t wave_total;   // planes of the whole wavefront
  uint32_t wave_start;   // planes of lower wavefronts
  uint32_t total;        // planes of the chunk
};

// The 256 lanes of a chunk are four consecutive wavefronts of the workgroup (which may hold
// more than one chunk).
__device__ __forceinline__ Places workgroup_places(uint32_t count, uint32_t* wave_totals) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t incl = wave_inclusive_sum(count, lane);
  if (lane == 63) wave_totals[wave] = incl;
  __syncthreads();
  Places p;
  p.in_wave = incl - count;
  p.wave_total = wave_totals[wave];
  p.wave_start = 0;
  p.total = 0;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const uint32_t t = wave_totals[(wave & ~3) + w];
    p.wave_start += w < (wave & 3) ? t : 0u;
    p.total += t;
  }
  return p;
}

// Span, within the wavefront's planes, of the half of its lanes that starts at lane 32*half.
__device__ __forceinline__ void half_span(const Places& p, int half, uint32_t& start, uint32_t& end) {
  const uint32_t middle = (uint32_t)__shfl((int)p.in_wave, 32);
  start = half ? middle : 0u;
  end = half ? p.wave_total : middle;
}

// Sum of the sizes of chunks 0..c-1, read from the table (run by one whole wavefront):
// 64 entries per pass, the lane's being the chunk at distance lane + 1 before c.  (Wider
// passes were slower: the polls of all workgroups in flight fall on the same few hundred
// table entries, and it is the number of these loads that costs.)  Returns false if a
// needed entry stayed empty for kSpinLimit polls, or if the stream has been marked flawed
// meanwhile (after one such failure nobody waits any more, so the launch ends at once).
__device__ bool bytes_before(uint64_t* table, const uint64_t* flaw, uint32_t c, int lane, uint64_t& before) {
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
      if ((polls & 255u) == 0u && __hip_atomic_load(flaw, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return false;
      __builtin_amdgcn_s_sleep(2);
    }
    sum += wave_sum64((uint32_t)lane <= first ? (s & zl::kValueMask) : 0ull);
    if (first != 64u) break;
    base -= 64;
  }
  before = sum;
  return true;
}

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// The lane's group of chunk c: words 1024*t + 4*tid .. +3 of the chunk, t = 0..7; words
// past the end of the message read as zero.  HALF: the message holds 16-bit words, which
// are coded as the 32-bit words v << 16.
template <bool HALF>
__device__ __forceinline__ void load_group(const void* __restrict__ message, size_t n, uint32_t c, int tid, uint32_t (&w)[32]) {
  const size_t base = (size_t)c * zl::kChunkWords;
  if constexpr (HALF) {
    const uint16_t* in = static_cast<const uint16_t*>(message);
    if (base + zl::kChunkWords <= n) {
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(in + base + 1024 * t + 4 * tid));
        w[4 * t] = v.x << 16; w[4 * t + 1] = v.x & 0xFFFF0000u; w[4 * t + 2] = v.y << 16; w[4 * t + 3] = v.y & 0xFFFF0000u;
      }
    } else {
#pragma unroll
      for (int j = 0; j < 32; ++j) {
        const size_t i = base + 1024 * (j >> 2) + 4 * tid + (j & 3);
        w[j] = i < n ? (uint32_t)in[i] << 16 : 0u;
      }
    }
  } else {
    const uint32_t* in = static_cast<const uint32_t*>(message);
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
  }
}

// The reverse; HALF keeps the upper halves of the words.
template <bool HALF>
__device__ __forceinline__ void store_group(void* __restrict__ message, size_t n, uint32_t c, int tid, const uint32_t (&w)[32]) {
  const size_t base = (size_t)c * zl::kChunkWords;
  if constexpr (HALF) {
    uint16_t* out = static_cast<uint16_t*>(message);
    if (base + zl::kChunkWords <= n) {
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const u32x2 v = {w[4 * t] >> 16 | (w[4 * t + 1] & 0xFFFF0000u), w[4 * t + 2] >> 16 | (w[4 * t + 3] & 0xFFFF0000u)};
        __builtin_nontemporal_store(v, reinterpret_cast<u32x2*>(out + base + 1024 * t + 4 * tid));
      }
    } else {
#pragma unroll
      for (int j = 0; j < 32; ++j) {
        const size_t i = base + 1024 * (j >> 2) + 4 * tid + (j & 3);
        if (i < n) out[i] = (uint16_t)(w[j] >> 16);
      }
    }
  } else {
    uint32_t* out = static_cast<uint32_t*>(message);
    if (base + zl::kChunkWords <= n) {
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const u32x4 v = {w[4 * t], w[4 * t + 1], w[4 * t + 2], w[4 * t + 3]};
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(out + base + 1024 * t + 4 * tid));
      }
    } else {
#pragma unroll
      for (int j = 0; j < 32; ++j) {
        const size_t i = base + 1024 * (j >> 2) + 4 * tid + (j & 3);
        if (i < n) out[i] = w[j];
      }
    }
  }
}

// A coded chunk that waits, in registers, for its place in the stream.
struct Coded {
  uint32_t planes[32];
  uint32_t reference, bitmap, chunk;
  Places at;
};

// CPW chunks per workgroup and counter value: chunks CPW*t .. CPW*t + CPW-1 are coded side
// by side by 256 lanes each, so that the counter, which serves one request in about 11.5 ns
// however many workgroups ask (measured: 32768 requests take 0.38 ms), is asked 1/CPW as often.
template <int CPW, bool HALF>
__global__ __launch_bounds__(kThreads * CPW, 4) void zl_compress_kernel(const void* __restrict__ in, size_t n, uint8_t* out,
                                                                        uint32_t chunks) {
  constexpr int kWaves = CPW * kThreads / 64;
  __shared__ uint32_t stage[kWaveStageWords * kWaves];
  __shared__ uint32_t wave_totals[kWaves];
  __shared__ uint32_t next_first;
  __shared__ uint64_t my_start[CPW];
  __shared__ uint32_t failed;
  Header* header = reinterpret_cast<Header*>(out);
  uint64_t* table = reinterpret_cast<uint64_t*>(out + zl::kHeaderBytes);
  uint8_t* payload = out + zl::kHeaderBytes + 8 * (size_t)chunks;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int part = tid / kThreads, lid = tid % kThreads;   // which of the CPW chunks, and the lane within it

  if (tid == 0) {
    next_first = CPW * __hip_atomic_fetch_add(&header->chunks, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    failed = 0;
  }
  __syncthreads();
  uint32_t first = next_first;
  if (first >= chunks) return;

  // A workgroup codes chunk after chunk.  A chunk's size is published as soon as it is
  // coded; its place is worked out, and it is written, only after the next chunk has
  // been coded in turn, by which time most of what its place depends on has arrived.
  // No wait for another workgroup lies between taking a counter value and publishing
  // the sizes of its chunks.
  constexpr uint32_t kNone = 0xFFFFFFFFu;
  Coded held;
  held.chunk = kNone;
  bool holding = false;
  for (;;) {
    const bool coding = first < chunks;   // the workgroup has chunks to code (its last ones may fall past the end)
    Coded now;
    now.chunk = kNone;
    if (coding) {
      const uint32_t c = first + part;
      const bool mine = c < chunks;
      uint32_t count = 0;
      if (mine) {
        load_group<HALF>(in, n, c, lid, now.planes);
        now.bitmap = zl::to_planes(now.planes, now.reference);
        now.chunk = c;
        count = (uint32_t)__builtin_popcount(now.bitmap);
      }
      now.at = workgroup_places(count, wave_totals);
      if (mine && lid == 0)
        __hip_atomic_store(&table[c], (c == 0 ? zl::kEnd : zl::kOwnSize) | (zl::kFixedChunkBytes + 4ull * now.at.total),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (holding) {
      const uint64_t bytes = zl::kFixedChunkBytes + 4ull * held.at.total;
      if ((wave & 3) == 0 && held.chunk != kNone) {   // the first wavefront of each chunk
        uint64_t before = 0;
        const bool ok = held.chunk == 0 || bytes_before(table, &header->flaw, held.chunk, lane, before);
        if (lane == 0) {
          if (!ok) {
            failed = 1;
            __hip_atomic_fetch_or(&header->flaw, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          }
          // publish a running total in any case, so that no later chunk waits for this one
          if (held.chunk != 0)
            __hip_atomic_store(&table[held.chunk], zl::kEnd | (before + bytes), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          my_start[part] = before;
        }
      }
      __syncthreads();
    }
    // the next counter value travels while the held chunks are written
    uint32_t asked = 0;
    if (coding && tid == 0) asked = CPW * __hip_atomic_fetch_add(&header->chunks, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (holding && held.chunk != kNone && !failed) {   // (a flawed stream is marked in the header; nothing more of it is written)
      uint32_t* dst = reinterpret_cast<uint32_t*>(payload + my_start[part]);
      dst[lid] = held.reference;
      dst[kThreads + lid] = held.bitmap;
      dst += 2 * kThreads + held.at.wave_start;
      // the wavefront's planes, 32 lanes at a time: into its LDS by lane, out of it by address
      // (LDS operations of one wavefront take effect in program order)
      uint32_t* mine = stage + kWaveStageWords * wave;
#pragma unroll 1
      for (int half = 0; half < 2; ++half) {
        uint32_t start, end;
        half_span(held.at, half, start, end);
        if ((lane >> 5) == half) {
          uint32_t pos = held.at.in_wave - start;
#pragma unroll
          for (int k = 0; k < 32; ++k)
            if ((held.bitmap >> k) & 1u) mine[staged(pos++)] = held.planes[k];
        }
        __builtin_amdgcn_wave_barrier();
        for (uint32_t i = lane; i < end - start; i += 64) dst[start + i] = mine[staged(i)];
        __builtin_amdgcn_wave_barrier();
      }
    }
    if (!coding) break;
    if (tid == 0) next_first = asked;
    held = now;
    holding = true;
    __syncthreads();
    first = next_first;
  }
}

// Completes the header once every chunk is placed (the chunk counter has run past its end).
__global__ void zl_finish_kernel(uint8_t* out, size_t n, uint32_t chunks) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  Header* header = reinterpret_cast<Header*>(out);
  const uint64_t* table = reinterpret_cast<const uint64_t*>(out + zl::kHeaderBytes);
  header->chunks = chunks;
  header->n = n;
  header->total = zl::kHeaderBytes + 8ull * chunks + (table[chunks - 1] & zl::kValueMask);
  header->magic = zl::kMagic;
}

// in_bytes: size of the buffer that holds the stream; every read stays below it.
template <bool HALF>
__global__ __launch_bounds__(kThreads) void zl_decompress_kernel(const uint8_t* __restrict__ in, size_t in_bytes, size_t n,
                                                                 void* __restrict__ out, uint32_t chunks) {
  __shared__ uint32_t stage[zl::kChunkWords + zl::kChunkWords / 32 + 64];   // spare words as in staged(); a lane may look one past its last plane
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
  // the chunk's plane words, as many as the span really holds: fetched by address before
  // anything is known about them, 32 loads in flight per lane
  const uint64_t held = words > 2 * kThreads ? words - 2 * kThreads : 0;
  const uint32_t stored = held < (uint64_t)zl::kChunkWords ? (uint32_t)held : (uint32_t)zl::kChunkWords;
  src += 2 * kThreads;
  // (a chunk that holds 16 planes per group or fewer, as every chunk of a 16-bit message does,
  // needs the first half of these loads and of the staging only; what a malformed stream then
  // picks up beyond its span is whatever the staging area held, which is as unspecified as
  // zeros would be)
  const bool upper_half = stored > 16u * kThreads;
  uint32_t p[32];
#pragma unroll
  for (int q = 0; q < 16; ++q) {
    const uint32_t i = tid + kThreads * q;
    p[q] = i < stored ? src[i] : 0u;
  }
  if (upper_half) {
#pragma unroll
    for (int q = 16; q < 32; ++q) {
      const uint32_t i = tid + kThreads * q;
      p[q] = i < stored ? src[i] : 0u;
    }
  }
  const Places at = workgroup_places((uint32_t)__builtin_popcount(bitmap), wave_totals);
#pragma unroll
  for (int q = 0; q < 16; ++q) stage[staged(tid + kThreads * q)] = p[q];
  if (upper_half) {
#pragma unroll
    for (int q = 16; q < 32; ++q) stage[staged(tid + kThreads * q)] = p[q];
  }
  __syncthreads();
  uint32_t pos = at.wave_start + at.in_wave;
  if constexpr (HALF) {
    // A stream made from 16-bit words has no planes below 16 and references with empty lower
    // halves.  Where that holds for every lane of the wavefront, only the upper 16 planes are
    // picked up and the lower ones are zeros the compiler can see, which takes a third off the
    // transpose as well; any other stream (arbitrary bytes) goes the general way below.
    const bool as_made = ((bitmap | reference) & 0xFFFFu) == 0u;
    if (__builtin_amdgcn_ballot_w64(!as_made) == 0) {
#pragma unroll
      for (int k = 0; k < 16; ++k) p[k] = 0u;
#pragma unroll
      for (int k = 16; k < 32; ++k) {
        const bool present = (bitmap >> k) & 1u;
        p[k] = present ? stage[staged(pos)] : 0u;
        pos += present ? 1u : 0u;
      }
      zl::from_planes(p, reference);
      store_group<HALF>(out, n, c, tid, p);
      return;
    }
  }
#pragma unroll
  for (int k = 0; k < 32; ++k) {
    const bool present = (bitmap >> k) & 1u;
    p[k] = present ? stage[staged(pos)] : 0u;
    pos += present ? 1u : 0u;
  }
  zl::from_planes(p, reference);
  store_group<HALF>(out, n, c, tid, p);
}

int compute_units() {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 256;
  return cus;
}

// 256-lane workgroups of the compress kernel per CU (wider workgroups: proportionally fewer).
// (Only a build with -DZC_TUNING_KNOBS lets ZL_WORKGROUPS_PER_CU override it.)
int workgroups_per_cu() {
#ifdef ZC_TUNING_KNOBS
  if (const char* e = getenv("ZL_WORKGROUPS_PER_CU")) {
    const int v = atoi(e);
    if (v >= 1 && v <= 64) return v;
  }
#endif
  return 4;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
constexpr size_t kMaxWords = (size_t)1 << 40;

size_t chunks_of(size_t n) { return (n + zl::kChunkWords - 1) / zl::kChunkWords; }

}  // namespace

namespace {
template <bool HALF>
int launch_zl_compress(const void* d_in, size_t n, void* d_out, size_t out_cap, void* stream) {
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
  constexpr int kPer = chunks_per_workgroup<HALF>();
  const size_t resident = (size_t)compute_units() * workgroups_per_cu() / kPer;   // 128 registers per lane: 16 wavefronts per CU
  const size_t tickets = (chunks + kPer - 1) / kPer;
  const unsigned grid = (unsigned)(tickets < resident ? tickets : resident);
  hipLaunchKernelGGL((zl_compress_kernel<kPer, HALF>), dim3(grid), dim3(kThreads * kPer), 0, s, d_in, n,
                     static_cast<uint8_t*>(d_out), (uint32_t)chunks);
  if (hipGetLastError() != hipSuccess) return ZC_ERR_LAUNCH;
  hipLaunchKernelGGL(zl_finish_kernel, dim3(1), dim3(64), 0, s, static_cast<uint8_t*>(d_out), n, (uint32_t)chunks);
  return hipGetLastError() == hipSuccess ? ZC_OK : ZC_ERR_LAUNCH;
}

template <bool HALF>
int launch_zl_decompress(const void* d_in, size_t in_bytes, size_t n, void* d_out, void* stream) {
  if (!d_in || (n && !d_out)) return ZC_ERR_NULL;
  if (!aligned16(d_in) || !aligned16(d_out)) return ZC_ERR_ALIGN;
  if (n > kMaxWords) return ZC_ERR_SIZE;
  const size_t chunks = chunks_of(n);
  if (in_bytes < zl::kHeaderBytes + 8 * chunks) return ZC_ERR_CAPACITY;
  if (chunks == 0) return ZC_OK;
  hipLaunchKernelGGL(zl_decompress_kernel<HALF>, dim3((unsigned)chunks), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                     static_cast<const uint8_t*>(d_in), in_bytes, n, d_out, (uint32_t)chunks);
  return hipGetLastError() == hipSuccess ? ZC_OK : ZC_ERR_LAUNCH;
}
}  // namespace

extern "C" {

size_t zl_max_compressed_size(size_t n) {
  if (n > kMaxWords) return 0;
  return zl::kHeaderBytes + chunks_of(n) * (size_t)(8 + zl::kFixedChunkBytes + 4 * zl::kChunkWords);
}

int zl_compress(const void* d_in, size_t n, void* d_out, size_t out_cap, void* stream) {
  return launch_zl_compress<false>(d_in, n, d_out, out_cap, stream);
}

int zl_compress16(const void* d_in, size_t n, void* d_out, size_t out_cap, void* stream) {
  return launch_zl_compress<true>(d_in, n, d_out, out_cap, stream);
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
  return launch_zl_decompress<false>(d_in, in_bytes, n, d_out, stream);
}

int zl_decompress16(const void* d_in, size_t in_bytes, size_t n, void* d_out, void* stream) {
  return launch_zl_decompress<true>(d_in, in_bytes, n, d_out, stream);
}

}  // extern "C"
