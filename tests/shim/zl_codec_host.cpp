// Host build of the per-lane pieces of the lossless codec (csrc/zl_codec.h), for checking
// them on the CPU against the reference.  Test-only.
#include <cstring>

#include "../../paper_2409_02423_amd/csrc/zl_codec.h"

extern "C" void zl_host_to_planes(const uint32_t* words, size_t groups, uint32_t* references, uint32_t* bitmaps,
                                  uint32_t* planes) {
  for (size_t g = 0; g < groups; ++g) {
    uint32_t w[32];
    std::memcpy(w, words + 32 * g, sizeof w);
    bitmaps[g] = zl::to_planes(w, references[g]);
    std::memcpy(planes + 32 * g, w, sizeof w);
  }
}

extern "C" void zl_host_from_planes(const uint32_t* planes, const uint32_t* references, size_t groups, uint32_t* words) {
  for (size_t g = 0; g < groups; ++g) {
    uint32_t p[32];
    std::memcpy(p, planes + 32 * g, sizeof p);
    zl::from_planes(p, references[g]);
    std::memcpy(words + 32 * g, p, sizeof p);
  }
}
