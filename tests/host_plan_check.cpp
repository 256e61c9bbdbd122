// Host-side check of the kernel-variant choice the GPU path shares between its host code and
// its mixed kernel (compiled with g++ by tests/test_host_logic.py): every shape gets a
// variant whose threads cover the whole channel within the kernels' limits.
#include <cstdint>
#include <cstdio>
#include <initializer_list>

#include "squant_plan.h"

using namespace squant;

int main() {
  long bad = 0, k9 = 0, k1 = 0, stream = 0, team = 0, generic = 0;
  for (int aligned = 0; aligned < 2; ++aligned)
    for (int64_t K : {1, 2, 4, 9, 25, 49})
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
          // no other admissible choice keeps the waves fuller
          for (int c : {1, 2, 4}) {
            const int64_t th = round_up64(N / c);
            if (th > 256 && c != 4) continue;
            bad += (N / c) * threads > (N / kpt) * th;
          }
        } else if (family == 1) {
          ++k1;
          const int nv = v == kK1x1 ? 1 : v == kK1x2 ? 2 : v == kK1x4 ? 4 : v == kK1x8 ? 8 : 0;
          if (nv == 0 || K != 1 || !aligned || N % 4 || N > kMaxK1Cin || N <= kMaxTeamCin) { ++bad; continue; }
          const int64_t nvec = N / 4, threads = round_up64((nvec + nv - 1) / nv);
          bad += threads * nv < nvec;
          bad += threads > (nv == 8 ? 1024 : 256);
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
        } else {
          ++generic;
          bad += v != kGeneric || work_items(130, N, K, 64, family) != 130;
          bad += aligned && K == 9 && N % 4 == 0 && N <= kMaxK9Cin;
          bad += aligned && K == 1 && N % 4 == 0;
        }
      }
  std::printf("plan_mismatches=%ld k9=%ld k1=%ld stream=%ld team=%ld generic=%ld\n", bad, k9, k1, stream, team, generic);
  return bad != 0;
}
