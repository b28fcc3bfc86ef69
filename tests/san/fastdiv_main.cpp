// Host check of the launch-constant division used by the kernels (gc_fastdiv.h): the multiply-shift
// form must equal x / d for every divisor the library can be given, on random and on edge dividends.
#include <cstdint>
#include <cstdio>
#include <random>

#include "../../paper_2506_17551_amd/csrc/gc_fastdiv.h"

int main() {
  std::mt19937_64 rng(20250617);
  long bad = 0, checked = 0;
  auto check = [&](uint32_t d, uint32_t x) {
    ++checked;
    if (gc::fast_div_host(x, gc::make_fastdiv(d)) != x / d) {
      if (bad < 10) std::printf("mismatch: %u / %u\n", x, d);
      ++bad;
    }
  };
  const uint32_t fixed[] = {1, 2, 3, 4, 5, 7, 8, 63, 64, 65, 100, 255, 256, 257, 1000, 1024, 2048, 4096, 4097,
                            5000, 8192, 10000, 65535, 65536, 65537, 70000, 1u << 20, (1u << 30) + 1, 0x7FFFFFFFu};
  for (uint32_t d : fixed) {
    for (uint32_t i = 0; i < 4096; ++i) {
      check(d, i);                   // small dividends
      check(d, 0xFFFFFFFFu - i);     // the top of the range
      const uint64_t mult = (uint64_t)i * d;
      if (mult <= 0xFFFFFFFFull) {   // around every multiple: the quotient steps exactly there
        check(d, (uint32_t)mult);
        if (mult > 0) check(d, (uint32_t)(mult - 1));
      }
    }
    for (int i = 0; i < 200000; ++i) check(d, (uint32_t)rng());
  }
  for (int k = 0; k < 200000; ++k) {
    const uint32_t d = (uint32_t)(rng() % 0x7FFFFFFFull) + 1u;
    for (int i = 0; i < 8; ++i) {
      const uint32_t x = (uint32_t)rng();
      check(d, x);
      const uint32_t m = (x / d) * d;
      check(d, m);
      if (m > 0) check(d, m - 1);
    }
  }
  std::printf("fastdiv host check: %ld divisions, %ld mismatches\n", checked, bad);
  return bad == 0 ? 0 : 1;
}
