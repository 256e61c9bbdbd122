// Which kernel variant a tensor's channels go through.  One function for the host, which
// sizes the launch from it, and for the mixed kernel, which picks the variant again per
// workgroup from the tensor's descriptor, so the two cannot disagree.
#pragma once

#include <stdint.h>

#include "squant_arith.h"  // SQ_HD

namespace squant {

enum Variant {
  kGeneric = 0,
  kK9x1 = 1, kK9x2 = 2, kK9x4 = 3,             // 3x3 kernels per thread: 1, 2, 4
  kK1x1 = 4, kK1x2 = 5, kK1x4 = 6, kK1x8 = 7,  // 1x1 / FC: 16-byte vectors per thread: 1, 2, 4, 8
  kK1Stream = 8,                               // 1x1 / FC beyond kMaxK1Cin: weights walked repeatedly
  kDw9 = 9,                                    // depthwise 3x3 (cin per group = 1): one thread per channel
  kK1Team = 10,                                // 1x1 / FC up to kMaxTeamCin: 4 to 16 channels per wave
  kK1x3 = 11, kK1x5 = 12, kK1x6 = 13, kK1x7 = 14,  // 1x1 / FC: 3, 5, 6, 7 vectors per thread
  kStream = 15,                                // any shape: nothing kept on chip, weights walked repeatedly
  kK1x16 = 16,                                 // 1x1 / FC: 16 vectors per thread
  kK1Wave = 32,                                // 1x1 / FC up to kMaxWaveCin, a wave per channel: kK1Wave + vectors per lane (2..8)
  kKs = 1024                                   // small kernels in registers: kKs + 4 * K + log2(kernels per thread)
};

constexpr int kMaxK9Cin = 4096;   // 3x3 variant: cin % 4 == 0 up to here
constexpr int kMaxK1Cin = 32768;  // 1x1 variant: cin % 4 == 0 up to here
constexpr int kMaxTeamCin = 256;  // 1x1 channels this short share a wave
constexpr int kMaxWaveCin = 2048; // 1x1 channels up to here take a wave each (at most 8 vectors per lane)
constexpr int kK1WaveSpan = 4;    // consecutive channels a wave of that kernel walks in a large launch (1 in others)
constexpr int kK1WaveThreads = 256;  // its workgroup in a launch of its own

SQ_HD int64_t round_up64(int64_t v) { return (v + 63) / 64 * 64; }

// Launch shape of the 1x1 / FC kernel for a channel of nvec 16-byte vectors (at most 8192):
// T threads of NV vectors each, NV in 1..8 or 16.  Candidates: workgroups of one or two waves
// or a whole multiple of four (which spread evenly over the four SIMDs of a compute unit) with
// NV = ceil(nvec / T) up to 8, and sixteen vectors in the fewest waves that cover the channel
// (up to four, else eight).  The score is the share of the T * NV vector slots in use (an idle
// vector still runs SQuant-E), weighted by what was measured on channels of 512 to 32768
// elements as a fraction of the HBM roofline: seven or eight vectors (80 VGPRs, six waves per
// SIMD) 0.85 of one to six or sixteen; 512 threads 0.95, 768 and 1024 threads 0.85 (the
// workgroup-wide steps of the channel stage run in more waves), sixteen vectors in 512 threads
// 0.90.  Ties go to the larger NV.  Examples: cin 3072 6 x 128 at 70 %, 4096 16 x 64 at 70 %,
// 8192 16 x 128 at 67 %, 16384 16 x 256 at 64 %, 24576 6 x 1024 at 55 %, 32768 16 x 512 at
// 56 % (8 x 1024, one workgroup per compute unit: 33 %); workgroups of 3, 5 to 7 or 9 to 15
// waves with up to eight vectors lose 10 to 25 points against their neighbours.
struct K1Shape { int nv; int threads; };
SQ_HD K1Shape k1_shape(int64_t nvec) {
  K1Shape best = {8, 1024};
  int64_t best_score = -1;
  auto consider = [&](int nv, int64_t T, int64_t weight) {
    if (nv * T < nvec) return;
    const int64_t score = nvec * weight * 1000 / (nv * T);
    if (score > best_score || (score == best_score && nv > best.nv)) {
      best_score = score;
      best.nv = nv;
      best.threads = (int)T;
    }
  };
  const int sizes[6] = {64, 128, 256, 512, 768, 1024};
  for (int i = 0; i < 6; ++i) {
    const int64_t T = sizes[i];
    const int64_t nv = (nvec + T - 1) / T;
    if (nv > 8) continue;
    consider((int)nv, T, (nv >= 7 ? 85 : 100) * (T >= 768 ? 85 : T == 512 ? 95 : 100));
  }
  const int64_t t16 = round_up64((nvec + 15) / 16);
  if (t16 <= 256) consider(16, t16, 100 * 100);
  else if (t16 <= 512) consider(16, 512, 100 * 90);
  return best;
}
SQ_HD int64_t k1_threads_for(int64_t nvec) { return k1_shape(nvec).threads; }
SQ_HD int k1_nv_for(int64_t nvec) { return k1_shape(nvec).nv; }
// Threads a 1x1 / FC channel of nvec vectors takes with nv vectors per thread.
SQ_HD int64_t k1_threads(int64_t nvec, int nv) {
  if (nv == k1_nv_for(nvec)) return k1_threads_for(nvec);
  return round_up64((nvec + nv - 1) / nv);
}

// The wave-per-channel 1x1 / FC kernel: 16-byte vectors per lane of a channel of N elements.
SQ_HD int k1_wave_nv(int64_t N) { return (int)((N / 4 + 63) / 64); }
SQ_HD bool is_k1_wave(int variant) { return variant >= kK1Wave + 2 && variant <= kK1Wave + 8; }

// 16-byte vectors per thread of a 1x1 / FC variant (0: not one), and back.
SQ_HD int k1_variant_nv(int variant) {
  switch (variant) {
    case kK1x1: return 1; case kK1x2: return 2; case kK1x3: return 3; case kK1x4: return 4;
    case kK1x5: return 5; case kK1x6: return 6; case kK1x7: return 7; case kK1x8: return 8;
    case kK1x16: return 16;
    default: return 0;
  }
}
SQ_HD int k1_variant_of(int nv) {
  const int v[9] = {kGeneric, kK1x1, kK1x2, kK1x3, kK1x4, kK1x5, kK1x6, kK1x7, kK1x8};
  return nv == 16 ? kK1x16 : v[nv];
}

// Small kernels held in registers (squant_ks.h): the kernel sizes it is built for, and the
// largest power of two (as its logarithm) of kernels one thread holds.
constexpr int kKsMaxK = 25;
SQ_HD bool ks_has(int64_t K) { return K == 2 || K == 3 || K == 4 || K == 5 || K == 7 || K == 25; }
SQ_HD constexpr int ks_max_kpt_log2(int64_t K) { return K <= 4 ? 3 : K <= 7 ? 2 : 0; }
// log2 of the kernels per thread for a channel of N such kernels: the largest power of two that
// divides N and puts the channel into ONE wave at least 60 % full, else the one that keeps the
// waves fullest (measured: a one-wave workgroup wins down to that fill - 1x7 with cin 192 and
// 1x3 with cin 384 10 % faster at 75 % than three full waves, 1x7 with cin 160 13 % faster at
// 62 % than at 83 %, cin 128 50 % slower at 50 % than at 100 % - while among workgroups of
// several waves the fullest wins by 11-13 %); only the largest one is built for workgroups
// beyond 256 threads.  -1: none fits (then the generic kernel takes the tensor).
SQ_HD int ks_kpt_log2(int64_t N, int64_t K) {
  if (!ks_has(K) || ((N * K) & 3) != 0) return -1;
  const int top = ks_max_kpt_log2(K);
  int best = -1;
  int64_t best_num = 0, best_den = 1;
  for (int lg = top; lg >= 0; --lg) {
    const int64_t c = (int64_t)1 << lg;
    if (N % c != 0) continue;
    const int64_t th = round_up64(N / c);
    if (th > 1024 || (th > 256 && lg != top)) continue;
    if (th == 64 && (N / c) * 10 >= th * 6) return lg;
    if ((N / c) * best_den > best_num * th) { best_num = N / c; best_den = th; best = lg; }
  }
  return best;
}
SQ_HD bool is_ks(int variant) { return variant >= kKs && variant < kKs + 4 * (kKsMaxK + 1); }
SQ_HD int ks_variant(int64_t K, int kpt_log2) { return kKs + 4 * (int)K + kpt_log2; }
SQ_HD int ks_variant_k(int variant) { return (variant - kKs) >> 2; }
SQ_HD int ks_variant_kpt(int variant) { return 1 << ((variant - kKs) & 3); }

// Kernel family of a tensor: 9 = the 3x3 kernel, 1 = the 1x1 / FC kernel, 2 = the streaming
// 1x1 / FC kernel, 3 = depthwise 3x3, 4 = short 1x1 / FC channels (several per wave), 5 = other
// small kernels in registers, 6 = 1x1 / FC channels that take a wave each, 0 = generic.
// aligned: weights on 16 bytes and output on 4 (what the vector loads / stores need)
SQ_HD int choose_family(int64_t N, int64_t K, bool aligned) {
  if (K == 9 && N == 1) return 3;  // any alignment: element-wise loads and stores
  if (K == 9 && (N & 3) == 0 && N <= kMaxK9Cin && aligned) return 9;
  if (K == 1 && (N & 3) == 0 && N <= kMaxTeamCin && aligned) return 4;
  if (K == 1 && (N & 3) == 0 && N <= kMaxWaveCin && aligned) return 6;
  if (K == 1 && (N & 3) == 0 && N <= kMaxK1Cin && aligned) return 1;
  if (K == 1 && (N & 3) == 0 && aligned) return 2;
  if (N > 1 && aligned && ks_kpt_log2(N, K) >= 0) return 5;
  return 0;
}

// The variant a tensor gets in a launch of its own.
SQ_HD int choose_variant(int64_t N, int64_t K, bool aligned) {
  const int family = choose_family(N, K, aligned);
  if (family == 9) {
    // kernels per thread: four when that puts the channel into one wave at least 60 % full
    // (cin 152..256; measured 11 % faster than three full waves at cin 160 and 192), else the
    // largest of 4, 2, 1 that keeps the waves fullest
    // (fill = (N / c) / round_up64(N / c), compared by cross-multiplication)
    int best_c = 4;
    int64_t best_num = 0, best_den = 1;
    for (int c = 4; c >= 1; c >>= 1) {
      const int64_t th = round_up64(N / c);
      if (th > 256 && c != 4) continue;
      const int64_t num = N / c;
      if (th == 64 && num * 10 >= th * 6) { best_c = c; break; }
      if (num * best_den > best_num * th) { best_num = num; best_den = th; best_c = c; }
    }
    return best_c == 4 ? kK9x4 : best_c == 2 ? kK9x2 : kK9x1;
  }
  if (family == 1) {
    return k1_variant_of(k1_nv_for(N / 4));
  }
  if (family == 2) return kK1Stream;
  if (family == 3) return kDw9;
  if (family == 4) return kK1Team;
  if (family == 6) return kK1Wave + k1_wave_nv(N);
  if (family == 5) return ks_variant(K, ks_kpt_log2(N, K));
  return kGeneric;
}

// Lanes that share a short 1x1 channel (see squant_k1_team.h).
SQ_HD int team_lanes(int64_t N) { return N <= 16 ? 4 : N <= 32 ? 8 : 16; }

// Workgroups a tensor of M output channels takes in a launch of T threads per workgroup:
// one per channel, except depthwise 3x3 (every thread has a channel of its own), short 1x1
// channels (one per team of lanes) and 1x1 channels of a wave each (wave_span per wave).  `family` as from choose_family.
SQ_HD int64_t work_items(int64_t M, int64_t N, int64_t K, int64_t T, int family, int wave_span) {
  if (family == 3) return (M + T - 1) / T;
  if (family == 4) { const int64_t per = T / team_lanes(N); return (M + per - 1) / per; }
  if (family == 6) { const int64_t per = T / 64 * wave_span; return (M + per - 1) / per; }
  (void)K;
  return M;
}

SQ_HD bool pointers_aligned(const void* w, const void* out) {
  return (reinterpret_cast<uintptr_t>(w) & 15u) == 0 && (reinterpret_cast<uintptr_t>(out) & 3u) == 0;
}

}  // namespace squant
