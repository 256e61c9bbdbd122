// SQuant reference solver -- TEST INFRASTRUCTURE ONLY.
//
// A plain, slow, single-purpose CPU implementation of the SQuant weight
// quantization solver (SQuant: On-the-Fly Data-Free Quantization via Diagonal
// Hessian Approximation, ICLR 2022).  It exists to define the expected output
// of the GPU library and is called only by the test-suite, the smoke check
// and the benchmark's CPU-baseline leg.  It shares no code with the GPU path
// and the product never routes through it.
//
// What it follows, per output channel m of a weight tensor W[M][N][K]
// (M output channels, N input channels = "kernels", K = kh*kw elements per
// kernel; Section 2.1 "Notations"):
//
//   scale      s_m = max|W[m]| / qmax          (Section 4: per-channel range;
//                                               Section 2.2 quantization formula)
//   SQuant-E   x = W/s_m, E = round(x), dE = E - x          (Algorithm 1, Eq. 5)
//   SQuant-K   per kernel: SQuantFlip(E, dE)                (Algorithm 1+2, Eq. 6)
//   update     per kernel: one flip candidate for SQuant-C  (Algorithm 3, App. B.3)
//   SQuant-C   per channel: SQuantFlip(K, dK)               (Algorithm 1+2, Eq. 7)
//
// Readings taken where the paper leaves a choice (all listed again in the
// design notes of the repository):
//   * arithmetic: x is one IEEE binary32 division, p = round(x) - x is exact in
//     binary32; p is then converted once to Q23 fixed point (P = rint(p*2^23))
//     and every sum / comparison is done on integers, so no result depends on
//     a summation order;
//   * round() is round-half-to-even; k = round(|e|) takes the FEWER flips on an
//     exact half (App. B.3 worked example: the SQuanted sum lies in (-0.5, 0.5]);
//   * top-k ties: lowest index first;
//   * x is clamped to [-qmax, qmax] before rounding (the clip of Section 2.2);
//   * all-zero channel: s_m = 1, codes 0;
//   * the accumulated perturbation of the channel-wise flip is the true sum of
//     all element perturbations of the channel after SQuant-K (Eq. 7), the
//     per-kernel candidates of Algorithm 3 being used for the sign filter and
//     the ranking only;
//   * Algorithm 3 "over SQuant": v is the perturbation of the k-th flipped
//     element AFTER its flip (0.5 <= |v| < 1); "under SQuant": the (k+1)-th
//     largest same-sign element, none if there is no such element; a kernel whose
//     sum is exactly 0 masks nothing and takes the largest |p| of either sign.
//
// Pins (tests/test_oracle_*.py): the flip figure's printed perturbations, the
// "3.2 -> 3 flips" and "+1.6 -> -0.4, candidate 2.7" worked examples, numpy for
// scales and plain rounding, exhaustive 2^K / 2^N flip search for the K and C
// stages, the constraints of Eq. 6 / 7 / 8, and the flipped-element counts of
// the appendix table (statistically).  Parity unpinned by the paper (pure
// conventions, see above): rounding ties, top-k ties, the exact-zero kernel, the
// 4-bit packing layout, and the batch-norm based activation range at the end of
// this file (the paper names the approach, prints no formula).
//
// Build: g++ -std=c++17 -O2 -fno-fast-math -ffp-contract=off -shared -fPIC -pthread

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <thread>
#include <vector>

namespace {

constexpr int32_t kOne = 1 << 23;   // 1.0 in Q23
constexpr int32_t kHalf = 1 << 22;  // 0.5 in Q23

enum Mode : int32_t { kModeE = 0, kModeEK = 1, kModeEKC = 2, kModeEC = 3 };

inline int sign_of(int64_t v) { return (v > 0) - (v < 0); }

// k = round(|e|) with an exact half rounded down (fewest flips).
inline int64_t flips_for(int64_t abs_sum) { return (abs_sum + kHalf - 1) >> 23; }

// Optional per-kernel / per-channel record of what the stages decided.
struct Trace {
  int32_t* kernel_k;     // [M*N] number of elements SQuant-K flipped
  int32_t* kernel_sum;   // [M*N] Q23 kernel perturbation sum after SQuant-K
  int32_t* cand_index;   // [M*N] element index of the SQuant-C candidate, -1 = none
  int32_t* cand_value;   // [M*N] Q23 perturbation of that element (0 = none)
  int64_t* channel_sum;  // [M]   Q23 channel perturbation sum after SQuant-K
  int32_t* channel_k;    // [M]   k of the channel-wise flip
  int32_t* perturbation; // [M*N*K] Q23 element perturbation after SQuant-K
};

// Indices of `p[0..n)` whose sign equals sgn, by |p| descending, index ascending.
std::vector<int32_t> ranked_same_sign(const int32_t* p, int32_t n, int sgn) {
  std::vector<int32_t> order;
  for (int32_t i = 0; i < n; ++i)
    if (sign_of(p[i]) == sgn) order.push_back(i);
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
    return std::abs(p[a]) > std::abs(p[b]);
  });
  return order;
}

// One output channel.  w: N*K floats; code: N*K int8 out; returns the scale.
float quantize_channel(const float* w, int32_t N, int32_t K, int32_t qmax, int32_t mode,
                       int8_t* code_out, const Trace* tr, int64_t m) {
  const int64_t len = (int64_t)N * K;

  // ---- scale: per-channel absmax over the symmetric grid [-qmax, qmax] ----
  float amax = 0.0f;
  for (int64_t j = 0; j < len; ++j) amax = std::fmax(amax, std::fabs(w[j]));
  std::vector<int32_t> c(len, 0), P(len, 0);
  float s = 1.0f;
  if (amax > 0.0f) {
    s = amax / (float)qmax;
    // ---- SQuant-E: scale, clip, round to nearest, element perturbation ----
    for (int64_t j = 0; j < len; ++j) {
      float x = w[j] / s;
      if (x > (float)qmax) x = (float)qmax;
      if (x < -(float)qmax) x = -(float)qmax;
      const float e = std::nearbyintf(x);
      const float p = e - x;  // exact in binary32
      c[j] = (int32_t)e;
      P[j] = (int32_t)std::lrintf(p * 8388608.0f);
    }
  }

  std::vector<int32_t> cand_i(N, -1), cand_v(N, 0);
  int64_t channel_sum = 0;

  if (mode != kModeE && amax > 0.0f) {
    for (int32_t n = 0; n < N; ++n) {
      int32_t* pk = &P[(int64_t)n * K];
      int32_t* ck = &c[(int64_t)n * K];
      int64_t e = 0;
      for (int32_t i = 0; i < K; ++i) e += pk[i];
      const int sgn = sign_of(e);
      const int64_t a = e < 0 ? -e : e;
      // ---- SQuant-K: flip the k largest same-sign perturbations ----
      const int64_t k = (mode == kModeEC) ? 0 : flips_for(a);
      std::vector<int32_t> L;
      if (sgn != 0) L = ranked_same_sign(pk, K, sgn);
      for (int64_t r = 0; r < k; ++r) {  // existence of k entries: App. B.1 proof
        const int32_t i = L[(size_t)r];
        ck[i] -= sgn;
        pk[i] -= sgn * kOne;
      }
      e -= (int64_t)sgn * k * kOne;
      channel_sum += e;
      // ---- perturbation update: the kernel's single SQuant-C candidate ----
      if (sgn == 0) {
        // nothing is masked: largest |p| of either sign, lowest index on ties
        int32_t best = -1, best_abs = 0;
        for (int32_t i = 0; i < K; ++i)
          if (std::abs(pk[i]) > best_abs) { best_abs = std::abs(pk[i]); best = i; }
        if (best >= 0) { cand_i[n] = best; cand_v[n] = pk[best]; }
      } else if (k * kOne > a) {  // over SQuant: the last flipped element, post-flip value
        const int32_t i = L[(size_t)(k - 1)];
        cand_i[n] = i;
        cand_v[n] = pk[i];
      } else if ((size_t)k < L.size()) {  // under SQuant: first un-flipped same-sign element
        const int32_t i = L[(size_t)k];
        cand_i[n] = i;
        cand_v[n] = pk[i];
      }
      if (tr) {
        const int64_t mn = m * N + n;
        if (tr->kernel_k) tr->kernel_k[mn] = (int32_t)k;
        if (tr->kernel_sum) tr->kernel_sum[mn] = (int32_t)e;
        if (tr->cand_index) tr->cand_index[mn] = cand_i[n];
        if (tr->cand_value) tr->cand_value[mn] = cand_v[n];
      }
    }
    if (tr && tr->perturbation)
      for (int64_t j = 0; j < len; ++j) tr->perturbation[m * len + j] = P[j];
    if (tr && tr->channel_sum) tr->channel_sum[m] = channel_sum;

    if (mode == kModeEKC || mode == kModeEC) {
      // ---- SQuant-C: flip the candidate of the k_c highest-ranked kernels ----
      const int sgn = sign_of(channel_sum);
      const int64_t a = channel_sum < 0 ? -channel_sum : channel_sum;
      const int64_t kc = flips_for(a);
      if (tr && tr->channel_k) tr->channel_k[m] = (int32_t)kc;
      if (sgn != 0 && kc > 0) {
        const std::vector<int32_t> LC = ranked_same_sign(cand_v.data(), N, sgn);
        const int64_t take = std::min<int64_t>(kc, (int64_t)LC.size());
        for (int64_t r = 0; r < take; ++r) {
          const int32_t n = LC[(size_t)r];
          c[(int64_t)n * K + cand_i[n]] -= sgn;
        }
      }
    }
  } else if (tr) {
    for (int32_t n = 0; n < N; ++n) {
      const int64_t mn = m * N + n;
      if (tr->kernel_k) tr->kernel_k[mn] = 0;
      if (tr->kernel_sum) tr->kernel_sum[mn] = 0;
      if (tr->cand_index) tr->cand_index[mn] = -1;
      if (tr->cand_value) tr->cand_value[mn] = 0;
    }
    if (tr->perturbation)
      for (int64_t j = 0; j < len; ++j) tr->perturbation[m * len + j] = P[j];
    if (tr->channel_sum) tr->channel_sum[m] = 0;
    if (tr->channel_k) tr->channel_k[m] = 0;
  }

  for (int64_t j = 0; j < len; ++j) code_out[j] = (int8_t)c[j];
  return s;
}

int check_args(const void* w, int32_t cout, int32_t cin, int32_t kh, int32_t kw, int32_t bits,
               int32_t mode, const void* codes, const void* scales) {
  if (!w || !codes || !scales) return 1;
  if (cout <= 0 || cin <= 0 || kh <= 0 || kw <= 0) return 2;
  if (bits < 2 || bits > 8) return 3;
  if (mode < 0 || mode > 3) return 4;
  return 0;
}

}  // namespace

extern "C" {

// Quantize one tensor W[cout][cin][kh][kw] (host pointers, synchronous).
// Returns 0, or 1 null pointer / 2 bad shape / 3 bad bits / 4 bad mode.
int squant_oracle_quantize(const float* w, int32_t cout, int32_t cin, int32_t kh, int32_t kw,
                           int32_t bits, int32_t mode, int8_t* codes, float* scales) {
  if (int rc = check_args(w, cout, cin, kh, kw, bits, mode, codes, scales)) return rc;
  const int32_t K = kh * kw, qmax = (1 << (bits - 1)) - 1;
  const int64_t len = (int64_t)cin * K;
  for (int64_t m = 0; m < cout; ++m)
    scales[m] = quantize_channel(w + m * len, cin, K, qmax, mode, codes + m * len, nullptr, m);
  return 0;
}

// Same result, output channels split statically over `threads` std::threads;
// the per-channel routine is unchanged.
int squant_oracle_quantize_mt(const float* w, int32_t cout, int32_t cin, int32_t kh, int32_t kw,
                              int32_t bits, int32_t mode, int8_t* codes, float* scales,
                              int32_t threads) {
  if (int rc = check_args(w, cout, cin, kh, kw, bits, mode, codes, scales)) return rc;
  if (threads < 1) threads = 1;
  const int32_t K = kh * kw, qmax = (1 << (bits - 1)) - 1;
  const int64_t len = (int64_t)cin * K;
  std::vector<std::thread> pool;
  for (int32_t t = 0; t < threads; ++t) {
    const int64_t lo = (int64_t)cout * t / threads, hi = (int64_t)cout * (t + 1) / threads;
    pool.emplace_back([=] {
      for (int64_t m = lo; m < hi; ++m)
        scales[m] = quantize_channel(w + m * len, cin, K, qmax, mode, codes + m * len, nullptr, m);
    });
  }
  for (auto& th : pool) th.join();
  return 0;
}

// Same result plus a record of the intermediate decisions.  Any trace pointer
// may be null.  Sizes: kernel_* and cand_* [cout*cin]; channel_* [cout];
// perturbation [cout*cin*kh*kw].  All perturbations are Q23 integers.
int squant_oracle_quantize_trace(const float* w, int32_t cout, int32_t cin, int32_t kh, int32_t kw,
                                 int32_t bits, int32_t mode, int8_t* codes, float* scales,
                                 int32_t* kernel_k, int32_t* kernel_sum, int32_t* cand_index,
                                 int32_t* cand_value, int64_t* channel_sum, int32_t* channel_k,
                                 int32_t* perturbation) {
  if (int rc = check_args(w, cout, cin, kh, kw, bits, mode, codes, scales)) return rc;
  const Trace tr{kernel_k, kernel_sum, cand_index, cand_value, channel_sum, channel_k, perturbation};
  const int32_t K = kh * kw, qmax = (1 << (bits - 1)) - 1;
  const int64_t len = (int64_t)cin * K;
  for (int64_t m = 0; m < cout; ++m)
    scales[m] = quantize_channel(w + m * len, cin, K, qmax, mode, codes + m * len, &tr, m);
  return 0;
}

int squant_oracle_hardware_threads(void) {
  const unsigned n = std::thread::hardware_concurrency();
  return n ? (int)n : 1;
}

// ---- output forms and input types beside the int8 codes of binary32 weights ----

// Two 4-bit codes to a byte (needs |code| <= 7, i.e. bits <= 4).  Row m of the output has
// (len + 1) / 2 bytes; byte j holds element 2j in its low nibble and element 2j + 1 in its
// high nibble, each as 4-bit two's complement; a missing last element leaves 0.
// Returns 0, or 1 null pointer / 2 bad shape / 3 a code outside [-8, 7].
int squant_oracle_pack_int4(const int8_t* codes, int64_t cout, int64_t len, uint8_t* packed) {
  if (!codes || !packed) return 1;
  if (cout <= 0 || len <= 0) return 2;
  const int64_t row = (len + 1) / 2;
  for (int64_t m = 0; m < cout; ++m)
    for (int64_t j = 0; j < row; ++j) {
      int nib[2] = {0, 0};
      for (int h = 0; h < 2; ++h) {
        const int64_t i = 2 * j + h;
        if (i >= len) continue;
        const int c = codes[m * len + i];
        if (c < -8 || c > 7) return 3;
        nib[h] = c < 0 ? c + 16 : c;  // two's complement in 4 bits
      }
      packed[m * row + j] = (uint8_t)(nib[0] + 16 * nib[1]);
    }
  return 0;
}

// The quantised weight of Section 2.2, code * scale of its output channel, as the one
// binary32 product (what Algorithm 1 returns).
int squant_oracle_dequantize(const int8_t* codes, const float* scales, int64_t cout, int64_t len,
                             float* out) {
  if (!codes || !scales || !out) return 1;
  if (cout <= 0 || len <= 0) return 2;
  for (int64_t m = 0; m < cout; ++m)
    for (int64_t i = 0; i < len; ++i) out[m * len + i] = (float)codes[m * len + i] * scales[m];
  return 0;
}

// The same product rounded to bfloat16 (the upper 16 bits of a binary32), round to nearest,
// ties to even: the two candidates are the binary32 value with its low 16 bits cleared and
// that plus one unit of the bfloat16 last place; the nearer one wins, an exact tie goes to
// the one whose last kept bit is 0.  Finite values only.
int squant_oracle_dequantize_bf16(const int8_t* codes, const float* scales, int64_t cout,
                                  int64_t len, uint16_t* out) {
  if (!codes || !scales || !out) return 1;
  if (cout <= 0 || len <= 0) return 2;
  for (int64_t m = 0; m < cout; ++m)
    for (int64_t i = 0; i < len; ++i) {
      const float v = (float)codes[m * len + i] * scales[m];
      uint32_t bits;
      std::memcpy(&bits, &v, 4);
      const uint32_t low = bits & 0xFFFFu;   // what is cut off
      uint32_t kept = bits >> 16;            // sign, exponent, 7 fraction bits
      if (low > 0x8000u || (low == 0x8000u && (kept & 1u))) kept += 1;  // magnitude grows either sign
      out[m * len + i] = (uint16_t)kept;
    }
  return 0;
}

// IEEE binary16 (1 sign, 5 exponent, 10 fraction bits) to binary32, exactly, from the
// format's definition: (-1)^s * 2^(e-15) * (1 + f/1024), subnormals 2^-14 * f/1024.
int squant_oracle_widen_f16(const uint16_t* h, int64_t n, float* out) {
  if (!h || !out) return 1;
  for (int64_t i = 0; i < n; ++i) {
    const int sign = h[i] >> 15, e = (h[i] >> 10) & 31, f = h[i] & 1023;
    double v;
    if (e == 31) v = f ? (double)NAN : (double)INFINITY;
    else if (e == 0) v = std::ldexp((double)f, -24);
    else v = std::ldexp(1024.0 + f, e - 25);
    out[i] = (float)(sign ? -v : v);
  }
  return 0;
}

// bfloat16 (1 sign, 8 exponent, 7 fraction bits: a binary32 cut after 16 bits) to binary32,
// from the same kind of definition: (-1)^s * 2^(e-127) * (1 + f/128), subnormals 2^-126 * f/128.
int squant_oracle_widen_bf16(const uint16_t* h, int64_t n, float* out) {
  if (!h || !out) return 1;
  for (int64_t i = 0; i < n; ++i) {
    const int sign = h[i] >> 15, e = (h[i] >> 7) & 255, f = h[i] & 127;
    double v;
    if (e == 255) v = f ? (double)NAN : (double)INFINITY;
    else if (e == 0) v = std::ldexp((double)f, -133);
    else v = std::ldexp(128.0 + f, e - 134);
    out[i] = (float)(sign ? -v : v);
  }
  return 0;
}

// ---- activation range without data (Section 4, experimental set-up) ----
// A batch-norm output channel c is taken as N(beta_c, gamma_c^2); the per-tensor range is
// the union over channels of beta_c -/+ n_sigma * |gamma_c|, cut at 0 from below when a ReLU
// follows, and the uniform quantizer on it has 2^bits levels.  binary32 throughout, one
// rounding per arithmetic step, in the order written here.  (The paper only names the
// approach - a wide batch-norm based range, clipped per tensor; n_sigma and the
// asymmetric quantizer are this library's reading.)
// out4 = {lo, hi, scale, zero_point as float}.  Returns 0, or 1 null / 2 bad size / 3 bad bits.
int squant_oracle_activation_range(const float* gamma, const float* beta, int64_t channels,
                                   float n_sigma, int32_t relu, int32_t bits, float* out4) {
  if (!gamma || !beta || !out4) return 1;
  if (channels <= 0) return 2;
  if (bits < 2 || bits > 16) return 3;
  float lo = INFINITY, hi = -INFINITY;
  for (int64_t c = 0; c < channels; ++c) {
    const float t = n_sigma * std::fabs(gamma[c]);
    const float a = beta[c] - t, b = beta[c] + t;
    if (a < lo) lo = a;
    if (b > hi) hi = b;
  }
  if (relu) {
    if (lo < 0.0f) lo = 0.0f;
    if (hi < 0.0f) hi = 0.0f;
  }
  lo += 0.0f;  // a zero bound is +0
  hi += 0.0f;
  const float q = (float)((1 << bits) - 1);
  const float span = hi - lo;
  const float scale = span > 0.0f ? span / q : 1.0f;
  float z = std::nearbyint(-lo / scale);
  if (z < 0.0f) z = 0.0f;
  if (z > q) z = q;
  out4[0] = lo; out4[1] = hi; out4[2] = scale; out4[3] = z;
  return 0;
}

}  // extern "C"
