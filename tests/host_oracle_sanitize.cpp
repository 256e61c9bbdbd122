// The CPU reference solver compiled together with this driver under the address and
// undefined-behaviour sanitizers (tests/test_host_logic.py): seeded random and degenerate
// tensors of assorted shapes through every mode and bit width, plus the packing, product and
// widening helpers.  Any out-of-bounds access, overflow or misaligned use aborts the run.
#include <cstdint>
#include <cstdio>
#include <vector>

#include "../oracle/squant_oracle.cpp"

static uint64_t g_rng = 0x2545F4914F6CDD1Dull;
static inline uint64_t xs() { g_rng ^= g_rng << 13; g_rng ^= g_rng >> 7; g_rng ^= g_rng << 17; return g_rng; }
static inline float unit() { return (float)((xs() >> 11) * (1.0 / 9007199254740992.0)) * 2.0f - 1.0f; }

int main() {
  const int shapes[][4] = {{1, 1, 1, 1}, {3, 1, 3, 3}, {4, 7, 3, 3}, {2, 64, 1, 1}, {5, 3, 7, 7},
                           {2, 33, 5, 5}, {6, 16, 3, 3}, {1, 1000, 1, 1}, {3, 5, 1, 3}};
  long runs = 0;
  for (const auto& sh : shapes) {
    const int64_t cout = sh[0], len = (int64_t)sh[1] * sh[2] * sh[3], total = cout * len;
    for (int kind = 0; kind < 4; ++kind) {
      std::vector<float> w((size_t)total);
      for (auto& v : w) {
        const float u = unit();
        v = kind == 0 ? u * 0.1f : kind == 1 ? (float)((int)(u * 8)) / 4.0f : kind == 2 ? 0.3f + 0.05f * u : 0.0f;
      }
      if (kind == 1 && total > 1) w[0] = 7.0f;
      std::vector<int8_t> codes((size_t)total);
      std::vector<float> scales((size_t)cout), deq((size_t)total);
      std::vector<uint8_t> packed((size_t)(cout * ((len + 1) / 2)));
      std::vector<uint16_t> deq16((size_t)total);
      for (int bits = 2; bits <= 8; ++bits)
        for (int mode = 0; mode < 4; ++mode) {
          if (squant_oracle_quantize(w.data(), sh[0], sh[1], sh[2], sh[3], bits, mode, codes.data(), scales.data())) return 2;
          if (squant_oracle_quantize_mt(w.data(), sh[0], sh[1], sh[2], sh[3], bits, mode, codes.data(), scales.data(), 3)) return 2;
          if (bits <= 4 && squant_oracle_pack_int4(codes.data(), cout, len, packed.data())) return 3;
          if (squant_oracle_dequantize(codes.data(), scales.data(), cout, len, deq.data())) return 4;
          if (squant_oracle_dequantize_bf16(codes.data(), scales.data(), cout, len, deq16.data())) return 4;
          ++runs;
        }
      std::vector<int32_t> kk((size_t)(cout * sh[1])), ks(kk.size()), ci(kk.size()), cv(kk.size()), ck((size_t)cout),
          pert((size_t)total);
      std::vector<int64_t> cs((size_t)cout);
      if (squant_oracle_quantize_trace(w.data(), sh[0], sh[1], sh[2], sh[3], 4, 2, codes.data(), scales.data(), kk.data(),
                                       ks.data(), ci.data(), cv.data(), cs.data(), ck.data(), pert.data()))
        return 5;
      float range[4];
      if (squant_oracle_activation_range(w.data(), w.data(), total, 6.0f, kind & 1, 8, range)) return 6;
    }
  }
  std::vector<uint16_t> h(65536);
  std::vector<float> f(65536);
  for (int i = 0; i < 65536; ++i) h[(size_t)i] = (uint16_t)i;
  if (squant_oracle_widen_f16(h.data(), 65536, f.data()) || squant_oracle_widen_bf16(h.data(), 65536, f.data())) return 7;
  std::printf("sanitized_runs=%ld\n", runs);
  return 0;
}
