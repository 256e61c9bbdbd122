// Host-side check of the GPU path's arithmetic building blocks (compiled with g++ by
// tests/test_host_logic.py): the top-5-of-9 selection network against std::sort on all
// 0/1 inputs and on random keys, and the reciprocal-based division against IEEE division on
// random operands, on operands built to sit as close as possible to a rounding midpoint,
// and on whole mantissa sweeps.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <functional>

#include "squant_arith.h"

static uint64_t g_rng = 0x9E3779B97F4A7C15ull;
static inline uint64_t xs() { g_rng ^= g_rng << 13; g_rng ^= g_rng >> 7; g_rng ^= g_rng << 17; return g_rng; }
static inline float f_from(uint32_t u) { float f; std::memcpy(&f, &u, 4); return f; }
static inline uint32_t u_from(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }
static uint64_t inv64(uint64_t a) { uint64_t x = a; for (int i = 0; i < 6; ++i) x *= 2 - a * x; return x; }

static long check_network() {
  long bad = 0;
  for (int bits = 0; bits < 512; ++bits) {
    int32_t s[9], ref[9];
    for (int i = 0; i < 9; ++i) s[i] = ref[i] = (bits >> i) & 1;
    std::sort(ref, ref + 9, std::greater<int32_t>());
    int32_t top[5];
    squant::top5_of_9(s, top);
    for (int i = 0; i < 5; ++i) bad += top[i] != ref[i];
  }
  for (int t = 0; t < 200000; ++t) {   // the unsigned network, keys across the sign bit
    uint32_t s[9], ref[9], top[5];
    for (int i = 0; i < 9; ++i) s[i] = ref[i] = (uint32_t)(xs() >> (t % 3 == 0 ? 61 : 32)) + 0x7ffffffcu;
    std::sort(ref, ref + 9, std::greater<uint32_t>());
    squant::top5_of_9u(s, top);
    for (int i = 0; i < 5; ++i) bad += top[i] != ref[i];
    uint32_t two[5];
    squant::Top9Rest rest;
    squant::top3_of_9u(s, two, rest);
    squant::next2_of_9u(rest, two);
    for (int i = 0; i < 5; ++i) bad += two[i] != ref[i];
  }
  for (int bits = 0; bits < 512; ++bits) {   // the two-part network on every 0/1 input
    uint32_t s[9], ref[9], two[5];
    for (int i = 0; i < 9; ++i) s[i] = ref[i] = (bits >> i) & 1;
    std::sort(ref, ref + 9, std::greater<uint32_t>());
    squant::Top9Rest rest;
    squant::top3_of_9u(s, two, rest);
    squant::next2_of_9u(rest, two);
    for (int i = 0; i < 5; ++i) bad += two[i] != ref[i];
    uint32_t top[5];
    squant::top5_of_9u(s, top);
    for (int i = 0; i < 5; ++i) bad += top[i] != ref[i];
  }
  for (uint32_t f = 0; f < 512; ++f) {  // flip bits to code bytes
    uint32_t b0, b1, b2;
    squant::spread_flip_bits(f, b0, b1, b2);
    for (int i = 0; i < 9; ++i) {
      const uint32_t got = i < 4 ? (b0 >> (8 * i)) & 255u : i < 8 ? (b1 >> (8 * (i - 4))) & 255u : b2;
      bad += got != ((f >> i) & 1u);
    }
  }
  for (int t = 0; t < 200000; ++t) {
    int32_t s[9], ref[9];
    for (int i = 0; i < 9; ++i) s[i] = ref[i] = (int32_t)(xs() >> (t % 3 == 0 ? 60 : 33)) - (1 << 29);
    std::sort(ref, ref + 9, std::greater<int32_t>());
    int32_t top[5];
    squant::top5_of_9(s, top);
    for (int i = 0; i < 5; ++i) bad += top[i] != ref[i];
  }
  return bad;
}

static long check_one(float w, float s) {
  const float r = 1.0f / s;
  return u_from(squant::div_by_reciprocal(w, s, r)) != u_from(w / s);
}

int main(int argc, char** argv) {
  const long n_random = argc > 1 ? std::atol(argv[1]) : 20000000;
  long bad_net = check_network();
  long bad_div = 0, n_div = 0;
  // random operands: divisor exponent in [-67, 60], quotient magnitude in [2^-27, 2^8]
  for (long i = 0; i < n_random; ++i) {
    const uint64_t a = xs(), b = xs();
    const int es = (int)(a % 128) - 67;
    uint32_t ms = (a >> 8) & 0x7fffff;
    if ((i & 15) == 0) ms = 0x7fffff - ((a >> 40) & 7);
    if ((i & 15) == 1) ms = (a >> 40) & 7;
    const float s = f_from(((uint32_t)(es + 127) << 23) | ms);
    const int ew = es + (int)(b % 36) - 27;
    const float w = f_from(((uint32_t)(ew + 127) << 23) | ((b >> 8) & 0x7fffff) | (uint32_t)((b >> 63) << 31));
    bad_div += check_one(w, s);
    ++n_div;
  }
  // quotients as close as possible to a midpoint between two floats:
  // W * 2^k = M * S + d with M an odd 25-bit integer and |d| small
  for (long i = 0; i < n_random / 8; ++i) {
    const uint64_t S = (xs() & 0x7fffff) | 0x800000 | 1;
    for (int k = 24; k <= 25; ++k)
      for (int d = -6; d <= 6; ++d) {
        if (!d) continue;
        const uint64_t mod = 1ull << k;
        const uint64_t M0 = ((uint64_t)(-(int64_t)d) * inv64(S)) & (mod - 1);
        for (uint64_t M = M0; M < (1ull << 25); M += mod) {
          if (M < (1ull << 24) || !(M & 1)) continue;
          const __int128 prod = (__int128)M * S + d;
          uint64_t W = (uint64_t)(prod >> k);
          if (((__int128)W << k) != prod) continue;
          while (W >= (1ull << 24) && !(W & 1)) W >>= 1;
          if (W >= (1ull << 24) || W < 1) continue;
          bad_div += check_one(std::ldexp((float)W, 3), std::ldexp((float)S, -20));
          bad_div += check_one(-std::ldexp((float)W, -40), std::ldexp((float)S, -60));
          n_div += 2;
        }
      }
  }
  // every numerator mantissa for a few divisors
  const uint32_t smants[] = {0, 1, 0x7fffff, 0x7ffffe, 0x400000, 0x3fffff, 0x555555, 0x2aaaaa, 0x123456};
  for (uint32_t sm : smants) {
    const float s = f_from((120u << 23) | sm);
    for (uint32_t m = 0; m < 0x800000; ++m) {
      bad_div += check_one(f_from((121u << 23) | m), s);
      ++n_div;
    }
  }
  std::printf("network_mismatches=%ld division_cases=%ld division_mismatches=%ld\n", bad_net, n_div, bad_div);
  return (bad_net || bad_div) ? 1 : 0;
}
