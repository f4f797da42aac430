// Division of a 31-bit unsigned number by a divisor fixed per launch, as one 64-bit multiply
// and a shift, so that the index decode of Section 3.3.3 (token index -> frame, row, column)
// runs on the scalar unit without a division sequence.  Host and device use the same code.
//
// For 1 <= d < 2^31 let s = ceil(log2 d) and m = floor(2^(31+s) / d) + 1 (m < 2^32).  Then
// floor(n / d) == (n * m) >> (31 + s) for every 0 <= n < 2^31 (round-up multiplier method:
// the error of m/2^(31+s) against 1/d is below 1/(d * 2^31), too small to carry n/d over the
// next integer while n < 2^31).
#pragma once
#include <stdint.h>

#if defined(__HIPCC__) || defined(__HIP__)
#define CROPE_HD __host__ __device__
#else
#define CROPE_HD
#endif

namespace crope {

struct FastDiv {
  uint32_t mul;
  uint32_t shift;   // 31 + s
  uint32_t d;
};

inline FastDiv make_fastdiv(uint32_t d) {   // 1 <= d < 2^31
  uint32_t s = 0;
  while (((uint64_t)1 << s) < d) ++s;
  FastDiv f;
  f.shift = 31 + s;
  f.mul = (uint32_t)((((uint64_t)1 << f.shift) / d) + 1);
  f.d = d;
  return f;
}

CROPE_HD inline uint32_t fastdiv(uint32_t n, const FastDiv& f) {   // n < 2^31
  return (uint32_t)(((uint64_t)n * f.mul) >> f.shift);
}

}  // namespace crope
