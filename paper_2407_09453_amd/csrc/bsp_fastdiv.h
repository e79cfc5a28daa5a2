// x / d by one multiply-high (library private; plain C++, also compiled on the host by the
// tests).  mul = floor(2^32 / d) + 1; the quotient floor(x * mul / 2^32) equals x / d while
// x * d < 2^32, which every launcher checks for the dividends it can produce.
#ifndef BSP_FASTDIV_H
#define BSP_FASTDIV_H

#include <stdint.h>

struct FastDiv {
  uint32_t d, mul;
};
inline FastDiv make_fastdiv(uint32_t d) {
  FastDiv f;
  f.d = d;
  f.mul = d > 1 ? (uint32_t)((0x100000000ull / d) + 1) : 0u;
  return f;
}
// the same arithmetic as the device's __umulhi
inline uint32_t fdiv_host(uint32_t x, FastDiv f) {
  return f.d == 1 ? x : (uint32_t)(((uint64_t)x * f.mul) >> 32);
}

#endif
