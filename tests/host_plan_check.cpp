// Host-side check of the kernel-variant choice the GPU path shares between its host code and
// its mixed kernel (compiled with g++ by tests/test_host_logic.py): every shape gets a
// variant whose threads cover the whole channel within the kernels' limits.
#include <cstdint>
#include <cstdio>
#include <initializer_list>

#include "squant_plan.h"

using namespace squant;

int main() {
  long bad = 0, k9 = 0, k1 = 0, stream = 0, team = 0, small = 0, generic = 0;
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
          if (nv == 0 || K != 1 || !aligned || N % 4 || N > kMaxK1Cin || N <= kMaxTeamCin) { ++bad; continue; }
          const int64_t nvec = N / 4, threads = k1_threads(nvec, nv);
          bad += threads * nv < nvec;
          bad += threads % 64 != 0 || threads > (nv == 8 ? 1024 : nv >= 5 && nv <= 6 ? 768 : 256);
          bad += k1_variant_of(nv) != v;
          if (nvec > 1024 && k1_wide_nv(nvec) <= 6) {
            // wide channels: five or six vectors per thread in 256, 512 or 768 threads
            bad += nv != k1_wide_nv(nvec) || nv < 5 || threads != k1_wide_threads(nvec) || threads % 256 != 0;
            continue;
          }
          // up to five vectors per thread while 256 threads suffice for that, else five to eight;
          // no admissible count of the class leaves fewer thread-vector slots idle
          if (nvec > 256 && nvec <= 448) {  // one wave of five to seven vectors per thread
            bad += nv != (nvec + 63) / 64 || threads != 64;
            continue;
          }
          bad += nvec <= 1024 ? nv > 5 : nv < 5;
          for (int c = (nvec <= 1024 ? 1 : 5); c <= (nvec <= 1024 ? 5 : 8) && nvec <= 2048; ++c) {
            const int64_t th = round_up64((nvec + c - 1) / c);
            if (th > 256) continue;
            bad += c * th < nv * threads;
          }
        } else if (family == 3) {
          bad += v != kDw9 || K != 9 || N != 1;
          bad += work_items(130, N, K, 64, family) != 3 || work_items(128, N, K, 64, family) != 2;
        } else if (family == 4) {
          ++team;  // short 1x1 channels: several per wave
          bad += v != kK1Team || K != 1 || !aligned || N % 4 || N > kMaxTeamCin;
          const int lanes = team_lanes(N);
          bad += (lanes != 4 && lanes != 8 && lanes != 16) || 64 % lanes != 0;
          bad += N > 4 * lanes * (lanes == 16 ? 4 : 1);           // vectors per lane: 1, or up to 4 at 16 lanes
          bad += work_items(130, N, K, 64, family) != (130 + 64 / lanes - 1) / (64 / lanes);
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
          bad += work_items(130, N, K, threads, family) != 130;
        } else {
          ++generic;
          bad += v != kGeneric || work_items(130, N, K, 64, family) != 130;
          bad += aligned && K == 9 && N % 4 == 0 && N <= kMaxK9Cin;
          bad += aligned && K == 1 && N % 4 == 0;
          bad += aligned && ks_has(K) && N > 1 && (N * K) % 4 == 0 && N <= 256;  // one kernel per thread always fits
        }
      }
  std::printf("plan_mismatches=%ld k9=%ld k1=%ld stream=%ld team=%ld small=%ld generic=%ld\n", bad, k9, k1, stream,
              team, small, generic);
  bad += small == 0;
  return bad != 0;
}
