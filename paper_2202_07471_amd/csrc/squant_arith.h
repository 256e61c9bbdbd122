// Pure arithmetic building blocks of the SQuant kernels that can also be compiled for
// the host, where the test-suite checks them exhaustively (no HIP headers needed).
#pragma once

#include <stdint.h>

#if defined(__HIPCC__)
#define SQ_HD __host__ __device__ __forceinline__
#else
#define SQ_HD inline
#endif

namespace squant {

// x = w / s, correctly rounded, from the correctly rounded reciprocal r = RN(1/s):
// q0 = RN(w r) is refined twice with the exact FMA residual w - q s.  The first step
// leaves a relative error below 2^-46 before its rounding, so q1 is a faithful
// rounding of w/s; Markstein's theorem (faithful quotient + correctly rounded
// reciprocal + exact residual => correctly rounded quotient) then makes q2 = RN(w/s).
// Needs the residuals to be exact, i.e. no underflow: callers use it only for
// 2^-60 <= max|w| <= 2^60, where an element small enough to underflow has |w/s| < 2^-30
// and rounds to code 0 / perturbation 0 either way.
SQ_HD float div_by_reciprocal(float w, float s, float r) {
  const float q0 = w * r;
  const float e0 = __builtin_fmaf(-q0, s, w);
  const float q1 = __builtin_fmaf(e0, r, q0);
  const float e1 = __builtin_fmaf(-q1, s, w);
  return __builtin_fmaf(e1, r, q1);
}

// compare-exchange: afterwards a >= b
#define SQ_CE(a, b)                                  \
  {                                                  \
    const int32_t hi_ = s[a] > s[b] ? s[a] : s[b];             \
    const int32_t lo_ = s[a] > s[b] ? s[b] : s[a];             \
    s[a] = hi_;                                      \
    s[b] = lo_;                                      \
  }

// Leaves the five largest of s[0..8] in s[0] >= s[1] >= ... >= s[4].  A 25-exchange
// sorting network for nine inputs with the three exchanges that only order the four
// smallest outputs removed; checked exhaustively on all 0/1 inputs by the test-suite.
SQ_HD void top5_of_9(int32_t (&s)[9]) {
  SQ_CE(0, 3) SQ_CE(1, 7) SQ_CE(2, 5) SQ_CE(4, 8)
  SQ_CE(0, 7) SQ_CE(2, 4) SQ_CE(3, 8) SQ_CE(5, 6)
  SQ_CE(0, 2) SQ_CE(1, 3) SQ_CE(4, 5) SQ_CE(7, 8)
  SQ_CE(1, 4) SQ_CE(3, 6) SQ_CE(5, 7)
  SQ_CE(0, 1) SQ_CE(2, 4) SQ_CE(3, 5)
  SQ_CE(2, 3) SQ_CE(4, 5)
  SQ_CE(1, 2) SQ_CE(3, 4)
}
#undef SQ_CE

}  // namespace squant
