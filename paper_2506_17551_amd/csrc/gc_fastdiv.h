// Exact unsigned 32-bit division by a divisor fixed for the launch, as a multiplication and two
// shifts (Granlund and Montgomery 1994, the round-up multiplier with an add-back): a pair's block is
// (pair number) / block, once per pair, and the hardware has no integer divide. Host part: the
// constants, and the same arithmetic in plain C++ for the host-side test; the device function
// fast_div lives beside the kernels.
#pragma once
#include <cstdint>

namespace gc {

struct FastDiv {
  uint32_t m, s1, s2;
};

inline FastDiv make_fastdiv(uint32_t d) {  // 1 <= d < 2^31
  uint32_t l = 0;
  while ((1ull << l) < d) ++l;
  FastDiv f;
  f.m = (uint32_t)((((1ull << l) - d) << 32) / d + 1ull);
  f.s1 = l < 1u ? l : 1u;
  f.s2 = l > 1u ? l - 1u : 0u;
  return f;
}

inline uint32_t fast_div_host(uint32_t x, FastDiv f) {  // what fast_div computes on the device
  const uint32_t t = (uint32_t)(((uint64_t)f.m * x) >> 32);
  return (t + ((x - t) >> f.s1)) >> f.s2;
}

}  // namespace gc
