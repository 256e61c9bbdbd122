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
// q0 = RN(w r), one exact-residual FMA e = RN(w - q0 s), one correction q1 = RN(q0 + e r).
// Before its last rounding q1 is within 2.01 * 2^-47 (relative) of w/s, so it can only be
// misrounded when w/s lies that close to a midpoint between two floats; the finitely many
// significand pairs for which it does are all enumerated and checked against IEEE division
// by the test-suite (tests/host_div_exhaustive.cpp), which makes q1 == RN(w/s) a checked
// fact rather than an estimate.  Needs the residual not to underflow: callers use it only
// for 2^-60 <= max|w| <= 2^60, where an element small enough to underflow has
// |w/s| < 2^-30 and rounds to code 0 / perturbation 0 either way.
SQ_HD float div_by_reciprocal(float w, float s, float r) {
  const float q0 = w * r;
  const float e0 = __builtin_fmaf(-q0, s, w);
  return __builtin_fmaf(e0, r, q0);
}

SQ_HD int32_t imax2(int32_t a, int32_t b) { return a > b ? a : b; }
SQ_HD int32_t imin2(int32_t a, int32_t b) { return a < b ? a : b; }
SQ_HD int32_t imax3(int32_t a, int32_t b, int32_t c) { return imax2(imax2(a, b), c); }
SQ_HD int32_t imin3(int32_t a, int32_t b, int32_t c) { return imin2(imin2(a, b), c); }
SQ_HD int32_t imed3(int32_t a, int32_t b, int32_t c) {
#if defined(__HIP_DEVICE_COMPILE__)  // the compiler does not form the instruction from min / max
  int32_t r;
  asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
#else
  return imax2(imin2(a, b), imin2(imax2(a, b), c));
#endif
}

// Leaves the five largest of x[0..8] in t[0] >= t[1] >= ... >= t[4], 25 three-input
// operations.  View x as a 3x3 matrix: sort the columns (9 ops), then the rows as far as
// needed (6 ops); rows and columns are then both ordered, so only
//   a b c
//   d e .
//   g . .
// can hold one of the five largest, a is the largest, e <= min(b, d), c <= b, g <= d.
// max/min(b, d) give ranks 2 and the runner-up D; c, e, g are sorted (3 ops) and D is
// inserted into them (5 ops).  Checked on every 0/1 input and on random keys by the
// test-suite (the operations are monotone, so the 0/1 principle applies).
SQ_HD void top5_of_9(const int32_t (&x)[9], int32_t (&t)[5]) {
  int32_t hi[3], mid[3], lo[3];
#pragma unroll
  for (int j = 0; j < 3; ++j) {
    hi[j] = imax3(x[j], x[j + 3], x[j + 6]);
    mid[j] = imed3(x[j], x[j + 3], x[j + 6]);
    lo[j] = imin3(x[j], x[j + 3], x[j + 6]);
  }
  const int32_t a = imax3(hi[0], hi[1], hi[2]);
  const int32_t b = imed3(hi[0], hi[1], hi[2]);
  const int32_t c = imin3(hi[0], hi[1], hi[2]);
  const int32_t d = imax3(mid[0], mid[1], mid[2]);
  const int32_t e = imed3(mid[0], mid[1], mid[2]);
  const int32_t g = imax3(lo[0], lo[1], lo[2]);
  const int32_t B = imax2(b, d), D = imin2(b, d);
  const int32_t C = imax3(c, e, g), E = imed3(c, e, g), G = imin3(c, e, g);
  const int32_t t1 = imin2(D, C), t2 = imin2(t1, E);
  t[0] = a;
  t[1] = B;
  t[2] = imax2(D, C);
  t[3] = imax2(t1, E);
  t[4] = imax2(t2, G);
}

// The same network on unsigned keys.
SQ_HD uint32_t umax2(uint32_t a, uint32_t b) { return a > b ? a : b; }
SQ_HD uint32_t umin2(uint32_t a, uint32_t b) { return a < b ? a : b; }
SQ_HD uint32_t umax3(uint32_t a, uint32_t b, uint32_t c) { return umax2(umax2(a, b), c); }
SQ_HD uint32_t umin3(uint32_t a, uint32_t b, uint32_t c) { return umin2(umin2(a, b), c); }
SQ_HD uint32_t umed3(uint32_t a, uint32_t b, uint32_t c) {
#if defined(__HIP_DEVICE_COMPILE__)
  uint32_t r;
  asm("v_med3_u32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
#else
  return umax2(umin2(a, b), umin2(umax2(a, b), c));
#endif
}
SQ_HD void top5_of_9u(const uint32_t (&x)[9], uint32_t (&t)[5]) {
  uint32_t hi[3], mid[3], lo[3];
#pragma unroll
  for (int j = 0; j < 3; ++j) {
    hi[j] = umax3(x[j], x[j + 3], x[j + 6]);
    mid[j] = umed3(x[j], x[j + 3], x[j + 6]);
    lo[j] = umin3(x[j], x[j + 3], x[j + 6]);
  }
  const uint32_t a = umax3(hi[0], hi[1], hi[2]);
  const uint32_t b = umed3(hi[0], hi[1], hi[2]);
  const uint32_t c = umin3(hi[0], hi[1], hi[2]);
  const uint32_t d = umax3(mid[0], mid[1], mid[2]);
  const uint32_t e = umed3(mid[0], mid[1], mid[2]);
  const uint32_t g = umax3(lo[0], lo[1], lo[2]);
  const uint32_t B = umax2(b, d), D = umin2(b, d);
  const uint32_t C = umax3(c, e, g), E = umed3(c, e, g), G = umin3(c, e, g);
  const uint32_t t1 = umin2(D, C), t2 = umin2(t1, E);
  t[0] = a;
  t[1] = B;
  t[2] = umax2(D, C);
  t[3] = umax2(t1, E);
  t[4] = umax2(t2, G);
}

// The network above in two parts: the three largest (19 operations), and the next two from
// what the first part leaves (6 operations) for the callers that need them.
struct Top9Rest { uint32_t c, e, g, D, C; };
SQ_HD void top3_of_9u(const uint32_t (&x)[9], uint32_t (&t)[5], Top9Rest& rest) {
  uint32_t hi[3], mid[3], lo[3];
#pragma unroll
  for (int j = 0; j < 3; ++j) {
    hi[j] = umax3(x[j], x[j + 3], x[j + 6]);
    mid[j] = umed3(x[j], x[j + 3], x[j + 6]);
    lo[j] = umin3(x[j], x[j + 3], x[j + 6]);
  }
  const uint32_t a = umax3(hi[0], hi[1], hi[2]);
  const uint32_t b = umed3(hi[0], hi[1], hi[2]);
  rest.c = umin3(hi[0], hi[1], hi[2]);
  const uint32_t d = umax3(mid[0], mid[1], mid[2]);
  rest.e = umed3(mid[0], mid[1], mid[2]);
  rest.g = umax3(lo[0], lo[1], lo[2]);
  rest.D = umin2(b, d);
  rest.C = umax3(rest.c, rest.e, rest.g);
  t[0] = a;
  t[1] = umax2(b, d);
  t[2] = umax2(rest.D, rest.C);
}
SQ_HD void next2_of_9u(const Top9Rest& rest, uint32_t (&t)[5]) {
  const uint32_t E = umed3(rest.c, rest.e, rest.g), G = umin3(rest.c, rest.e, rest.g);
  const uint32_t t1 = umin2(rest.D, rest.C), t2 = umin2(t1, E);
  t[3] = umax2(t1, E);
  t[4] = umax2(t2, G);
}

// Bits 0..8 of f (one per element of a 3x3 kernel) as 0/1 bytes in the layout of the
// kernel's packed codes: b0 = elements 0-3, b1 = elements 4-7, b2 = element 8.  A 4-bit
// field times 0x204081 puts bit i at positions i, i + 7, i + 14, i + 21, of which
// 0, 8, 16, 24 are kept: bit i in byte i.
SQ_HD void spread_flip_bits(uint32_t f, uint32_t& b0, uint32_t& b1, uint32_t& b2) {
  b0 = ((f & 15u) * 0x204081u) & 0x01010101u;
  b1 = (((f >> 4) & 15u) * 0x204081u) & 0x01010101u;
  b2 = (f >> 8) & 1u;
}

}  // namespace squant
