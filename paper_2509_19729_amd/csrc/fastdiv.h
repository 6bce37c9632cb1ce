// Division of a 32-bit unsigned value by a divisor fixed at launch time, done as
// multiply-high plus two shifts (the round-up multiplier method of Granlund and
// Montgomery, "Division by invariant integers using multiplication", 1994).
// Exact for every n in [0, 2^32) and every divisor in [1, 2^32).
#pragma once
#include <stdint.h>

struct FastDiv {
  uint32_t d;      // the divisor
  uint32_t magic;  // floor(2^32 (2^l - d) / d) + 1, l = ceil(log2 d)
  uint32_t sh1;    // min(l, 1)
  uint32_t sh2;    // max(l - 1, 0)
};

inline FastDiv make_fastdiv(uint32_t d) {
  FastDiv f;
  f.d = d;
  uint32_t l = 0;
  while (l < 32 && (uint64_t(1) << l) < d) ++l;
  f.magic = uint32_t((((uint64_t(1) << l) - d) << 32) / d + 1);
  f.sh1 = l < 1 ? l : 1;
  f.sh2 = l > 0 ? l - 1 : 0;
  return f;
}

#if defined(__HIPCC__)
__device__ __forceinline__ uint32_t fd_div(uint32_t n, const FastDiv& f) {
  const uint32_t t = __umulhi(f.magic, n);
  return (t + ((n - t) >> f.sh1)) >> f.sh2;
}
#endif

// Same arithmetic with a 64-bit product, for host-side checks of the constants.
inline uint32_t fd_div_host(uint32_t n, const FastDiv& f) {
  const uint32_t t = uint32_t((uint64_t(f.magic) * n) >> 32);
  return (t + ((n - t) >> f.sh1)) >> f.sh2;
}
