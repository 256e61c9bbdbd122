// Exhaustive check of the short reciprocal division used by the GPU path:
//     r = RN(1/s);  q0 = RN(w r);  e = RN(w - q0 s) (one FMA);  q1 = RN(q0 + e r) (one FMA)
// claim: q1 == RN(w/s) for all binary32 w, s (no underflow/overflow in the intermediates).
//
// Why a finite enumeration proves it.  Exponents do not matter, so take the 24-bit integer
// significands W, S in [2^23, 2^24).  Before its final rounding q1 is
//     v = w/s + (w/s - q0) eps_r + (RN(e) - e) r,       |eps_r| <= 2^-24,
// and with |w/s - q0| <= (w/s)(2^-23 + 2^-48), |e| <= w (2^-23 + 2^-48), |RN(e) - e| <= 2^-24 |e|
// this gives |v - w/s| < 2.01 * 2^-47 (w/s).  q1 can differ from RN(w/s) only if a rounding
// midpoint lies between v and w/s.  Midpoints are M / 2^k with M odd in [2^24, 2^25) and
// k = 25 (W < S) or k = 24 (W >= S), and  w/s - M/2^k = d / (S 2^k)  with the integer
// d = W 2^k - M S != 0; relative to w/s that is |d| / (W 2^k) >= |d| 2^-49 (k = 25) or
// |d| 2^-48 (k = 24).  So only |d| <= 8 (k = 25) or |d| <= 4 (k = 24) can go wrong.  Every
// (W, S, M) with |d| <= 12 is enumerated below (M S = -d mod 2^k solved for M, every
// solution when S is even) and checked against IEEE division.
//
// Build: g++ -O2 -mfma -ffp-contract=off -fopenmp
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>

#include "squant_arith.h"

static inline uint32_t bits_of(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }
static uint64_t inv_odd(uint64_t a) { uint64_t x = a; for (int i = 0; i < 6; ++i) x *= 2 - a * x; return x; }

int main() {
  long long checked = 0, bad = 0;
#pragma omp parallel for schedule(dynamic, 4096) reduction(+ : checked, bad)
  for (int64_t S = 1ll << 23; S < (1ll << 24); ++S) {
    const int j = __builtin_ctzll((uint64_t)S);     // S = 2^j * Sodd
    const uint64_t Sodd = (uint64_t)S >> j, Sinv = inv_odd(Sodd);
    const float s = (float)S, r = 1.0f / s;
    for (int k = 24; k <= 25; ++k) {
      for (int d = -12; d <= 12; ++d) {
        if (d == 0 || (d & ((1 << j) - 1))) continue;            // need 2^j | d
        const int kk = k - j;                                     // M Sodd = -(d / 2^j) mod 2^kk
        if (kk <= 0) continue;
        const uint64_t mod = 1ull << kk;
        const uint64_t m0 = ((uint64_t)(-(int64_t)(d >> j)) * Sinv) & (mod - 1);
        for (uint64_t M = m0; M < (1ull << 25); M += mod) {
          if (M < (1ull << 24) || !(M & 1)) continue;
          const __int128 num = (__int128)M * S + d;               // = W 2^k
          if (num & (((__int128)1 << k) - 1)) continue;
          const uint64_t W = (uint64_t)(num >> k);
          if (W < (1ull << 23) || W >= (1ull << 24)) continue;
          const float w = (float)W;
          const float got = squant::div_by_reciprocal(w, s, r);
          ++checked;
          if (bits_of(got) != bits_of(w / s)) {
#pragma omp critical
            if (bad < 5) std::printf("mismatch W=%llu S=%lld d=%d k=%d\n", (unsigned long long)W, (long long)S, d, k);
            ++bad;
          }
        }
      }
    }
  }
  std::printf("near_midpoint_cases=%lld mismatches=%lld\n", checked, bad);
  return bad ? 1 : 0;
}
