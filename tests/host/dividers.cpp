// Host check of the multiply-high dividers the kernels use for tile and work-group indices
// (fast_div_setup in csrc/wino_kernels.hpp): for every divisor tried, the prepared pair must
// reproduce n / d at the values of n where a wrong constant shows first (multiples of d and their
// neighbours, the largest index 2^30 - 1) and on a pseudo-random sample.  A wrong quotient would
// send a kernel to another tile's addresses, so this is checked without a GPU.
// Prints "ok <divisors> <checks>" and exits 0, or the first failure and exits 1.
#include <cstdint>
#include <cstdio>

#include "wino_kernels.hpp"

// what the device function computes: the high word of n * mul (or n itself), shifted
static uint32_t divide(uint32_t n, uint32_t mul, uint32_t sh) {
  return (mul ? (uint32_t)(((uint64_t)n * mul) >> 32) : n) >> sh;
}

int main() {
  const uint32_t top = (1u << 30) - 1;
  uint64_t checks = 0, divisors = 0;
  uint64_t state = 0x9E3779B97F4A7C15ull;
  auto next = [&]() {
    state ^= state << 13, state ^= state >> 7, state ^= state << 17;
    return state;
  };
  auto check_divisor = [&](uint32_t d) -> bool {
    uint32_t mul, sh;
    wino::fast_div_setup(d, &mul, &sh);
    ++divisors;
    auto one = [&](uint32_t n) -> bool {
      ++checks;
      if (divide(n, mul, sh) == n / d) return true;
      std::printf("d = %u, n = %u: got %u, want %u (mul %u, shift %u)\n", d, n, divide(n, mul, sh),
                  n / d, mul, sh);
      return false;
    };
    if (!one(0) || !one(top) || !one(top - 1)) return false;
    // multiples of d and their neighbours: the first few, the last few, and a spread between
    const uint32_t kmax = top / d;
    for (uint32_t i = 0; i < 64; ++i) {
      const uint32_t ks[3] = {i <= kmax ? i : kmax, kmax - (i <= kmax ? i : 0),
                              (uint32_t)(next() % ((uint64_t)kmax + 1))};
      for (uint32_t k : ks) {
        const uint64_t at = (uint64_t)k * d;
        if (at <= top && !one((uint32_t)at)) return false;
        if (at >= 1 && at - 1 <= top && !one((uint32_t)(at - 1))) return false;
        if (at + 1 <= top && !one((uint32_t)(at + 1))) return false;
        if (at + d - 1 <= top && !one((uint32_t)(at + d - 1))) return false;
      }
    }
    for (int i = 0; i < 256; ++i)
      if (!one((uint32_t)(next() & top))) return false;
    return true;
  };
  for (uint32_t d = 1; d <= 70000; ++d)            // every small divisor (tiles per row / image, chunks)
    if (!check_divisor(d)) return 1;
  for (uint32_t f = 16; f <= 29; ++f)              // around every power of two up to 2^30
    for (int32_t o = -3; o <= 3; ++o)
      if (!check_divisor((1u << f) + (uint32_t)o)) return 1;
  for (int i = 0; i < 20000; ++i)                  // a sample of large divisors
    if (!check_divisor((uint32_t)(next() % top) + 1)) return 1;
  if (!check_divisor(top) || !check_divisor(1u << 30)) return 1;
  std::printf("ok %llu %llu\n", (unsigned long long)divisors, (unsigned long long)checks);
  return 0;
}
