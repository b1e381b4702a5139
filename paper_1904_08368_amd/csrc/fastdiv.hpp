// Division of a non-negative 31-bit integer by a divisor known on the host: one multiply-high
// and one shift on the device instead of the ~25-instruction software division (the kernel
// prologues divide by tile counts and image extents; a workgroup lives for only a few thousand
// instructions).
//   d == 1:  n / d = n
//   d >= 2:  l = ceil(log2 d), mul = floor(2^(31+l) / d) + 1, n / d = mulhi(n, mul) >> (l - 1)
// exact for 0 <= n < 2^31 (round-up method: mul*d - 2^(31+l) lies in (0, d], and d <= 2^l).
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define RELAY_HD __host__ __device__
#else
#define RELAY_HD
#endif

namespace relay {

struct FastDiv {
  uint32_t mul;    // 0: the divisor is 1
  uint32_t shift;
};

inline FastDiv make_fastdiv(uint32_t d) {
  FastDiv f{0u, 0u};
  if (d <= 1) return f;
  uint32_t l = 0;
  while ((1ull << l) < d) ++l;
  f.mul = (uint32_t)(((1ull << (31 + l)) / d) + 1ull);
  f.shift = l - 1;
  return f;
}

RELAY_HD inline uint32_t fast_div(uint32_t n, FastDiv f) {
  return f.mul ? (uint32_t)(((uint64_t)n * f.mul) >> 32) >> f.shift : n;
}

}  // namespace relay
