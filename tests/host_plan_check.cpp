// Host-side check of the kernel-variant choice the GPU path shares between its host code and
// its mixed kernel (compiled with g++ by tests/test_host_logic.py): every shape gets a
// variant whose threads cover the whole channel within the kernels' limits.
#include <cstdint>
#include <cstdio>
#include <initializer_list>

#include "squant_plan.h"

using namespace squant;

int main() {
  long bad = 0, k9 = 0, k1 = 0, stream = 0, team = 0, wave = 0, small = 0, generic = 0;
  // 1x1 / FC launch shapes: the measured optima
  const struct { int64_t cin; int nv, threads; } optima[] = {
      {512, 2, 64},     {1024, 4, 64},    {3072, 6, 128},    {4096, 16, 64},   {5120, 5, 256},   {8192, 16, 128},
      {12288, 16, 192}, {16384, 16, 256}, {24576, 6, 1024}, {28672, 16, 512}, {32768, 16, 512}};
  for (const auto& o : optima) {
    const K1Shape sh = k1_shape(o.cin / 4);
    bad += sh.nv != o.nv || sh.threads != o.threads;
  }
  for (int aligned = 0; aligned < 2; ++aligned)
    for (int64_t K : {1, 2, 3, 4, 5, 6, 7, 8, 9, 25, 49})
      for (int64_t N = 1; N <= 40000; N += (N < 600 ? 1 : 61)) {
        const int family = choose_family(N, K, aligned != 0);
        const int v = choose_variant(N, K, aligned != 0);
        if (family == 9) {
          ++k9;
          const int kpt = v == kK9x4 ? 4 : v == kK9x2 ? 2 : v == kK9x1 ? 1 : 0;
          if (kpt == 0 || K != 9 || !aligned || N % 4 || N > kMaxK9Cin) { ++bad; continue; }
          const int64_t threads = round_up64(N / kpt);
          bad += N % kpt != 0;               // every thread owns whole kernels
          bad += threads * kpt < N;          // all kernels covered
          bad += threads > 1024;
          bad += kpt != 4 && threads > 256;  // the narrow variants are built for 256 threads
          // one wave at least 60 % full with four kernels per thread, else no other admissible
          // choice keeps the waves fuller
          if (round_up64(N / 4) == 64 && (N / 4) * 10 >= 64 * 6) {
            bad += kpt != 4;
          } else {
            for (int c : {1, 2, 4}) {
              const int64_t th = round_up64(N / c);
              if (th > 256 && c != 4) continue;
              bad += (N / c) * threads > (N / kpt) * th;
            }
          }
        } else if (family == 1) {
          ++k1;
          const int nv = k1_variant_nv(v);
          if (nv == 0 || K != 1 || !aligned || N % 4 || N > kMaxK1Cin || N <= kMaxWaveCin) { ++bad; continue; }
          const int64_t nvec = N / 4, threads = k1_threads(nvec, nv);
          bad += threads * nv < nvec;
          bad += k1_variant_of(nv) != v;
          // eight or fewer vectors in one or two waves or a multiple of four, or sixteen vectors
          // in any whole waves up to four, or eight
          bad += !((nv >= 1 && nv <= 8) || nv == 16);
          if (nv <= 8) {
            bad += !(threads == 64 || threads == 128 || (threads % 256 == 0 && threads <= 1024));
            bad += nv != (nvec + threads - 1) / threads;  // no thread without a vector of its own
          } else {
            bad += threads % 64 != 0 || (threads > 256 && threads != 512);
          }
        } else if (family == 6) {
          ++wave;  // 1x1 channels that take a wave each
          bad += !is_k1_wave(v) || K != 1 || !aligned || N % 4 || N <= kMaxTeamCin || N > kMaxWaveCin;
          const int nv = v - kK1Wave;
          bad += nv != k1_wave_nv(N) || nv < 2 || nv > 8 || 64 * nv * 4 < N;
          bad += work_items(130, N, K, 256, family, kK1WaveSpan) != (130 + 4 * kK1WaveSpan - 1) / (4 * kK1WaveSpan);
          bad += work_items(130, N, K, 64, family, 1) != 130;
        } else if (family == 3) {
          bad += v != kDw9 || K != 9 || N != 1;
          bad += work_items(130, N, K, 64, family, 1) != 3 || work_items(128, N, K, 64, family, 1) != 2;
        } else if (family == 4) {
          ++team;  // short 1x1 channels: several per wave
          bad += v != kK1Team || K != 1 || !aligned || N % 4 || N > kMaxTeamCin;
          const int lanes = team_lanes(N);
          bad += (lanes != 4 && lanes != 8 && lanes != 16) || 64 % lanes != 0;
          bad += N > 4 * lanes * (lanes == 16 ? 4 : 1);           // vectors per lane: 1, or up to 4 at 16 lanes
          bad += work_items(130, N, K, 64, family, 1) != (130 + 64 / lanes - 1) / (64 / lanes);
        } else if (family == 2) {
          ++stream;  // a 1x1 channel too long for the register-resident kernel
          bad += v != kK1Stream || K != 1 || !aligned || N % 4 || N <= kMaxK1Cin;
        } else if (family == 5) {
          ++small;  // other small kernels in registers
          if (!is_ks(v) || !aligned || !ks_has(K) || (N * K) % 4 || N < 2 || K > kKsMaxK) { ++bad; continue; }
          const int kpt = ks_variant_kpt(v), top = 1 << ks_max_kpt_log2(K);
          bad += ks_variant_k(v) != K || v != ks_variant(K, ks_kpt_log2(N, K));
          bad += kpt < 1 || kpt > top || (kpt & (kpt - 1)) != 0;
          bad += N % kpt != 0;                 // every thread owns whole kernels
          const int64_t threads = round_up64(N / kpt);
          bad += threads * kpt < N || threads > 1024;
          bad += kpt != top && threads > 256;  // only the largest is built for 1024 threads
          bad += K * kpt > 32 && kpt > 1;      // elements a thread holds in registers
          bool roomy = false;                  // some admissible choice is one wave at least 60 % full
          for (int c = 1; c <= top; c *= 2) {
            if (N % c) continue;
            const int64_t th = round_up64(N / c);
            if (th > 1024 || (th > 256 && c != top)) continue;
            const bool ok60 = th == 64 && (N / c) * 10 >= th * 6;
            roomy |= ok60;
            bad += ok60 && c > kpt;            // the largest such count is the one taken
          }
          if (roomy) {
            bad += (N / kpt) * 10 < threads * 6;
          } else {                             // else none keeps the waves fuller
            for (int c = 1; c <= top; c *= 2) {
              if (N % c) continue;
              const int64_t th = round_up64(N / c);
              if (th > 1024 || (th > 256 && c != top)) continue;
              bad += (N / c) * threads > (N / kpt) * th;
            }
          }
          bad += work_items(130, N, K, threads, family, 1) != 130;
        } else {
          ++generic;
          bad += v != kGeneric || work_items(130, N, K, 64, family, 1) != 130;
          bad += aligned && K == 9 && N % 4 == 0 && N <= kMaxK9Cin;
          bad += aligned && K == 1 && N % 4 == 0;
          bad += aligned && ks_has(K) && N > 1 && (N * K) % 4 == 0 && N <= 256;  // one kernel per thread always fits
        }
      }
  std::printf("plan_mismatches=%ld k9=%ld k1=%ld stream=%ld team=%ld wave=%ld small=%ld generic=%ld\n", bad, k9, k1,
              stream, team, wave, small, generic);
  bad += small == 0 || wave == 0;
  return bad != 0;
}
