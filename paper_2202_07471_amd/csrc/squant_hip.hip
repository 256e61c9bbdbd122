// SQuant weight-quantization solver, gfx950 (MI355X) kernels and C ABI.
//
// One workgroup owns one output channel from the first byte read to the last
// byte written: the channel's weights are read from HBM once (into registers
// for 3x3 and 1x1 kernels, into LDS otherwise), the absmax scale, rounding
// (SQuant-E), kernel-wise flip (SQuant-K), candidate update (Algorithm 3) and
// channel-wise flip (SQuant-C) all run on chip, and only the codes and one
// float scale go back to HBM.  Perturbations are Q23 integers, so every sum is
// order independent.  This file is the host side: argument checks, the choice
// of kernel variant per tensor, the grouping of a batch into launches.
//
// Section / algorithm numbers refer to "SQuant: On-the-Fly Data-Free
// Quantization via Diagonal Hessian Approximation" (ICLR 2022).

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <vector>

#include "squant.h"

#include "squant_common.h"
#include "squant_generic.h"
#include "squant_k9.h"
#include "squant_ks.h"
#include "squant_k1.h"
#include "squant_k1_wave.h"
#include "squant_mixed.h"
#include "squant_stream.h"
#include "squant_act.h"
#include "squant_plan.h"

namespace {

using namespace squant;

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------

struct DeviceLimits { int lds_bytes; bool ok; };

DeviceLimits device_limits() {
  int dev = 0, lds = 0;
  if (hipGetDevice(&dev) != hipSuccess) return {0, false};
  if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess)
    return {0, false};
  return {lds, true};
}

constexpr int kStaticLds = 16 * 4 + 16 * 8 + 256 * 4 + 16 + 64;  // static __shared__ of the kernels, padded

size_t generic_lds_bytes(int64_t N, int64_t K) {
  const int64_t L = N * K;
  return (size_t)(4 * L + (K == 1 ? 0 : 8 * N) + ((L + 3) & ~(int64_t)3) + 16);
}

int generic_threads(int64_t N, int64_t K) {
  const int64_t L = N * K;
  int64_t want = (K == 1) ? (L + 7) / 8 : (K >= kWaveKernelMinK) ? N * kWave : N;
  want = (want + kWave - 1) / kWave * kWave;
  return (int)std::min<int64_t>(512, std::max<int64_t>(kWave, want));
}

int check_common(int32_t bits, int mode) {
  if (bits < 2 || bits > 8) return SQUANT_ERR_BITS;
  if (mode < SQUANT_MODE_E || mode > SQUANT_MODE_EC) return SQUANT_ERR_MODE;
  return SQUANT_OK;
}

// Weight type and output format; `out` may be null when only the enums are checked.
int check_format(int wtype, int output, int32_t bits, const void* w, const void* out) {
  if (wtype < SQUANT_W_F32 || wtype > SQUANT_W_BF16) return SQUANT_ERR_FORMAT;
  if (output < SQUANT_OUT_INT8 || output > SQUANT_OUT_BF16) return SQUANT_ERR_FORMAT;
  if (output == SQUANT_OUT_INT4 && bits > 4) return SQUANT_ERR_BITS;
  const uintptr_t wmask = wtype == SQUANT_W_F32 ? 3u : 1u;
  if (reinterpret_cast<uintptr_t>(w) & wmask) return SQUANT_ERR_FORMAT;
  if (output == SQUANT_OUT_F32 && (reinterpret_cast<uintptr_t>(out) & 3u)) return SQUANT_ERR_FORMAT;
  if (output == SQUANT_OUT_BF16 && (reinterpret_cast<uintptr_t>(out) & 1u)) return SQUANT_ERR_FORMAT;
  return SQUANT_OK;
}

int check_shape(int32_t cout, int32_t cin, int32_t kh, int32_t kw) {
  if (cout <= 0 || cin <= 0 || kh <= 0 || kw <= 0) return SQUANT_ERR_SHAPE;
  const int64_t K = (int64_t)kh * kw;
  const int64_t L = K * cin;
  if (K > (1 << 20) || L > (int64_t)1 << 30) return SQUANT_ERR_SHAPE;
  return SQUANT_OK;
}

constexpr int kMixed = 100;      // Group::variant of a launch of squant_channel_mixed
constexpr int kMixedWave = 101;  // the same for the tensors whose channels take one wave each
constexpr int kKsMixed = 102;    // Group::variant of a launch of squant_channel_ks_mixed
constexpr int kKsMixedMaxThreads = 128;

struct Group {
  int variant;
  int threads;
  size_t lds;
  std::vector<TensorDesc> t;
  bool fixed_threads = false;  // mixed launch: a non-generic member has set the workgroup size
  bool wave_members = false;   // holds wave-per-channel 1x1 tensors: LDS for a selection area per wave
};

// threads / lds: of a launch of the tensor's own variant.  mix_threads: what the tensor needs as
// a member of a mixed launch (0: it cannot join one), where the per-thread work follows the
// launch's workgroup size.
struct Plan { int variant; int threads; size_t lds; int mix_threads; };

inline size_t round_up(size_t v, size_t to) { return (v + to - 1) / to * to; }

// The fallback that takes any channel: nothing is kept on chip.
Plan stream_plan(int64_t N) {
  const int th = (int)std::min<int64_t>(kStreamThreads, std::max<int64_t>(2 * kWave, round_up64(N)));
  return Plan{kStream, th, 16, 0};  // no dynamic LDS; 16 stands for "fits"
}

// Picks the kernel variant and launch shape for one tensor (every tensor fits one).
Plan plan_tensor(const void* w, const void* out, int64_t N, int64_t K, int lds_limit) {
  const int variant = choose_variant(N, K, pointers_aligned(w, out));
  // LDS: a selection area per wave of the launch's workgroup, added when the launch goes out
  if (is_k1_wave(variant)) return Plan{variant, kK1WaveThreads, 16, kWave};
  switch (variant) {
    case kK9x1: case kK9x2: case kK9x4: {
      const int kpt = variant == kK9x4 ? 4 : variant == kK9x2 ? 2 : 1;
      // LDS: the channel's int8 codes
      const int th = (int)round_up64(N / kpt);
      return Plan{variant, th, round_up((size_t)9 * N, 16), th};
    }
    case kK1x1: case kK1x2: case kK1x3: case kK1x4: case kK1x5: case kK1x6: case kK1x7: case kK1x8:
    case kK1x16: {
      const int nv = k1_variant_nv(variant);
      const int64_t nvec = N / 4;
      const int th = (int)k1_threads(nvec, nv);
      // the mixed kernel carries the routines of up to four vectors per thread
      const int mix = nv <= 4 ? th : nvec <= 4 * kMixedMaxThreads ? (int)round_up64((nvec + 3) / 4) : 0;
      // LDS: the owners' masks, a word per thread (of the launch's workgroup, which a mixed
      // launch may make larger), two with sixteen vectors
      const size_t lds = nv > 8 ? (size_t)8 * th : (size_t)4 * std::max(th, kMixedMaxThreads);
      return Plan{variant, th, lds, mix};
    }
    case kDw9: return Plan{kDw9, kWave, 16, kWave};     // no LDS; 16 stands for "fits"
    case kK1Team: return Plan{kK1Team, kWave, 16, kWave};
    case kK1Stream: {
      const size_t lds = round_up((size_t)N, 16);  // the channel's int8 codes
      if (lds + sizeof(K9Shared) + 64 > (size_t)lds_limit) return stream_plan(N);
      return Plan{kK1Stream, 1024, lds, 0};
    }
    default: break;
  }
  if (is_ks(variant))  // LDS: the channel's int8 codes
    return Plan{variant, (int)round_up64(N / ks_variant_kpt(variant)), round_up((size_t)K * N, 16), 0};
  const size_t lds = generic_lds_bytes(N, K);
  if (lds + kStaticLds > (size_t)lds_limit) return stream_plan(N);
  const int th = generic_threads(N, K);
  return Plan{kGeneric, th, lds, th};
}

// Whether a tensor may join a launch of the mixed kernel: the mixed kernel carries a routine
// for it that fits its workgroup size and LDS.
bool mixable(const Plan& p, size_t lds_cap) {
  return p.mix_threads > 0 && p.mix_threads <= kMixedMaxThreads &&
         p.lds <= lds_cap;
}

typedef void (*kernel_t)(LaunchArgs);

// The small-kernel variant's instantiation for (K, kernels per thread), workgroup size and mode.
template <int K, int KPT>
kernel_t ks_kernel_of(int threads, int mode, bool largest) {
#define SQ_KS_ROW(T)                                                                          \
  {squant_channel_ks<T, SQUANT_MODE_E, K, KPT>, squant_channel_ks<T, SQUANT_MODE_EK, K, KPT>, \
   squant_channel_ks<T, SQUANT_MODE_EKC, K, KPT>, squant_channel_ks<T, SQUANT_MODE_EC, K, KPT>}
  static const kernel_t small[4] = SQ_KS_ROW(256);
  if (threads <= 256 || !largest) return small[mode];
  if constexpr (KPT == (1 << ks_max_kpt_log2(K))) {
    static const kernel_t large[4] = SQ_KS_ROW(1024);
    return large[mode];
  }
#undef SQ_KS_ROW
  return small[mode];
}
template <int K>
kernel_t ks_kernel_k(int kpt, int threads, int mode) {
  const bool largest = kpt == (1 << ks_max_kpt_log2(K));
  constexpr int top = 1 << ks_max_kpt_log2(K);
  if (kpt == 1) return ks_kernel_of<K, 1>(threads, mode, largest);
  if constexpr (top >= 2) if (kpt == 2) return ks_kernel_of<K, 2>(threads, mode, largest);
  if constexpr (top >= 4) if (kpt == 4) return ks_kernel_of<K, 4>(threads, mode, largest);
  if constexpr (top >= 8) if (kpt == 8) return ks_kernel_of<K, 8>(threads, mode, largest);
  return nullptr;
}
kernel_t ks_kernel(int variant, int threads, int mode) {
  const int kpt = ks_variant_kpt(variant);
  switch (ks_variant_k(variant)) {
    case 2: return ks_kernel_k<2>(kpt, threads, mode);
    case 3: return ks_kernel_k<3>(kpt, threads, mode);
    case 4: return ks_kernel_k<4>(kpt, threads, mode);
    case 5: return ks_kernel_k<5>(kpt, threads, mode);
    case 7: return ks_kernel_k<7>(kpt, threads, mode);
    case 25: return ks_kernel_k<25>(kpt, threads, mode);
    default: return nullptr;
  }
}

// Launches tensors [begin, end) of a group (at most kInlineDescs of them) as one kernel.
int launch_part(const Group& g, size_t begin, size_t end, int qmax, int mode, int output, int wtype,
                int wave_span, hipStream_t st) {
  LaunchArgs a{};
  int64_t total = 0;
  bool uniform = true;
  auto items_of = [&](const TensorDesc& t) {
    return work_items(t.M, t.N, t.K, g.threads, choose_family(t.N, t.K, pointers_aligned(t.w, t.out)),
                      wave_span);
  };
  const int64_t items0 = items_of(g.t[begin]);
  for (size_t i = begin; i < end; ++i) {
    const TensorDesc& t = g.t[i];
    const int64_t items = items_of(t);
    a.table[i - begin] = t;
    a.table[i - begin].first = (int32_t)total;  // first workgroup within this launch
    total += items;
    uniform &= items == items0;
    if (total > 0x7fffffff) return SQUANT_ERR_SHAPE;
  }
  if (total <= 0) return SQUANT_ERR_SHAPE;
  a.n_tensors = (int)(end - begin);
  a.total = (int32_t)total;
  a.uniform_m = uniform ? (int32_t)items0 : 0;
  a.uniform_shift = -1;
  if (uniform && (items0 & (items0 - 1)) == 0)
    for (int sh = 0; sh < 31; ++sh)
      if (((int64_t)1 << sh) == items0) a.uniform_shift = sh;
  a.qmax = qmax;
  a.mode = mode;
  a.out_format = output;
  a.wtype = wtype;
  a.wave_span = wave_span;
#define SQ_K9_ROW(T, KPT)                                                                     \
  {squant_channel_k9<T, SQUANT_MODE_E, KPT>, squant_channel_k9<T, SQUANT_MODE_EK, KPT>,       \
   squant_channel_k9<T, SQUANT_MODE_EKC, KPT>, squant_channel_k9<T, SQUANT_MODE_EC, KPT>}
  static const kernel_t k9x1[4] = SQ_K9_ROW(256, 1);
  static const kernel_t k9x2[4] = SQ_K9_ROW(256, 2);
  static const kernel_t k9x4[4] = SQ_K9_ROW(256, 4);
  static const kernel_t k9x4_large[4] = SQ_K9_ROW(1024, 4);
#undef SQ_K9_ROW
  // four kernels per thread in workgroups of exactly two waves (cin 260 .. 512) or one
  // (cin 152 .. 256): weight type and wave count compiled in
#define SQ_K9_ROW_X(WT, NWC)                                                                  \
  {squant_channel_k9<256, SQUANT_MODE_E, 4, WT, NWC>, squant_channel_k9<256, SQUANT_MODE_EK, 4, WT, NWC>, \
   squant_channel_k9<256, SQUANT_MODE_EKC, 4, WT, NWC>, squant_channel_k9<256, SQUANT_MODE_EC, 4, WT, NWC>}
  static const kernel_t k9x4_two_waves[3][4] = {SQ_K9_ROW_X(SQUANT_W_F32, 2), SQ_K9_ROW_X(SQUANT_W_F16, 2),
                                                SQ_K9_ROW_X(SQUANT_W_BF16, 2)};
  static const kernel_t k9x4_one_wave[4] = SQ_K9_ROW_X(SQUANT_W_F32, 1);
#undef SQ_K9_ROW_X
#define SQ_K1_ROW(NV)                                                                         \
  {squant_channel_k1<SQUANT_MODE_E, NV>, squant_channel_k1<SQUANT_MODE_E, NV>,                \
   squant_channel_k1<SQUANT_MODE_EKC, NV>, squant_channel_k1<SQUANT_MODE_EKC, NV>}
  // (for one-element kernels E&K equals E and E&C equals E&K&C)
  static const kernel_t k1[8][4] = {SQ_K1_ROW(1), SQ_K1_ROW(2), SQ_K1_ROW(3), SQ_K1_ROW(4),
                                    SQ_K1_ROW(5), SQ_K1_ROW(6), SQ_K1_ROW(7), SQ_K1_ROW(8)};
  static const kernel_t k1x16[4] = SQ_K1_ROW(16);
#define SQ_K1W_ROW(NV)                                                                        \
  {squant_channel_k1_wave<SQUANT_MODE_E, NV>, squant_channel_k1_wave<SQUANT_MODE_E, NV>,      \
   squant_channel_k1_wave<SQUANT_MODE_EKC, NV>, squant_channel_k1_wave<SQUANT_MODE_EKC, NV>}
  static const kernel_t k1w[7][4] = {SQ_K1W_ROW(2), SQ_K1W_ROW(3), SQ_K1W_ROW(4), SQ_K1W_ROW(5),
                                     SQ_K1W_ROW(6), SQ_K1W_ROW(7), SQ_K1W_ROW(8)};
#undef SQ_K1W_ROW
#undef SQ_K1_ROW
  static const kernel_t k1s[4] = {squant_channel_k1_stream<SQUANT_MODE_E>, squant_channel_k1_stream<SQUANT_MODE_E>,
                                  squant_channel_k1_stream<SQUANT_MODE_EKC>, squant_channel_k1_stream<SQUANT_MODE_EKC>};
  static const kernel_t stream[4] = {squant_channel_stream<SQUANT_MODE_E>, squant_channel_stream<SQUANT_MODE_EK>,
                                     squant_channel_stream<SQUANT_MODE_EKC>, squant_channel_stream<SQUANT_MODE_EC>};
  static const kernel_t k1team[4] = {squant_channel_k1_team<SQUANT_MODE_E>, squant_channel_k1_team<SQUANT_MODE_E>,
                                     squant_channel_k1_team<SQUANT_MODE_EKC>, squant_channel_k1_team<SQUANT_MODE_EKC>};
  static const kernel_t dw9[4] = {squant_channel_dw9<SQUANT_MODE_E>, squant_channel_dw9<SQUANT_MODE_EK>,
                                  squant_channel_dw9<SQUANT_MODE_EKC>, squant_channel_dw9<SQUANT_MODE_EC>};
  static const kernel_t mixed[4] = {squant_channel_mixed<SQUANT_MODE_E>, squant_channel_mixed<SQUANT_MODE_EK>,
                                    squant_channel_mixed<SQUANT_MODE_EKC>, squant_channel_mixed<SQUANT_MODE_EC>};
  static const kernel_t ksmixed[4] = {squant_channel_ks_mixed<SQUANT_MODE_E>, squant_channel_ks_mixed<SQUANT_MODE_EK>,
                                      squant_channel_ks_mixed<SQUANT_MODE_EKC>, squant_channel_ks_mixed<SQUANT_MODE_EC>};
  const kernel_t kernel = is_ks(g.variant) ? ks_kernel(g.variant, g.threads, mode)
                          : g.variant == kKsMixed ? ksmixed[mode]
                          : (g.variant == kMixed || g.variant == kMixedWave) ? mixed[mode]
                          : g.variant == kK1x16 ? k1x16[mode]
                          : is_k1_wave(g.variant) ? k1w[g.variant - kK1Wave - 2][mode]
                          : k1_variant_nv(g.variant) ? k1[k1_variant_nv(g.variant) - 1][mode]
                          : g.variant == kK1Stream ? k1s[mode]
                          : g.variant == kStream ? stream[mode]
                          : g.variant == kDw9 ? dw9[mode]
                          : g.variant == kK1Team ? k1team[mode]
                          : g.variant == kK9x1 ? k9x1[mode]
                          : g.variant == kK9x2 ? k9x2[mode]
                          : g.variant == kK9x4 ? (g.threads == 2 * kWave ? k9x4_two_waves[wtype][mode]
                                                  : g.threads == kWave && wtype == SQUANT_W_F32 ? k9x4_one_wave[mode]
                                                  : g.threads <= 256 ? k9x4[mode] : k9x4_large[mode])
                                               : squant_channel_generic;
  if (!kernel) return SQUANT_ERR_UNSUPPORTED;
  size_t lds = g.lds;
  if (g.wave_members) lds = std::max(lds, (size_t)(g.threads / kWave) * sizeof(K1WaveSel));
  if (lds > 48 * 1024) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
      (void)hipGetLastError();
      return SQUANT_ERR_DEVICE;
    }
  }
  const unsigned grid = (unsigned)total;
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(g.threads), g.variant == kStream ? 0 : lds, st, a);
  if (hipGetLastError() != hipSuccess) return SQUANT_ERR_DEVICE;
  return SQUANT_OK;
}

// A group goes out in launches of at most kInlineDescs tensors each.
int launch_group(const Group& g, int qmax, int mode, int output, int wtype, hipStream_t st) {
  // Waves of the wave-per-channel 1x1 kernel walk several channels each where that still
  // leaves the chip (8192 resident waves) a few rounds of them; in a mixed launch one.
  int wave_span = 1;
  if (is_k1_wave(g.variant)) {
    int64_t channels = 0;
    for (const auto& t : g.t) channels += t.M;
    if (channels >= (int64_t)kK1WaveSpan * 2 * 8192) wave_span = kK1WaveSpan;
  }
  for (size_t begin = 0; begin < g.t.size(); begin += kInlineDescs) {
    const size_t end = std::min(g.t.size(), begin + (size_t)kInlineDescs);
    if (int rc = launch_part(g, begin, end, qmax, mode, output, wtype, wave_span, st)) return rc;
  }
  return SQUANT_OK;
}

}  // namespace

extern "C" {

int squant_quantize_ex(const void* d_w, squant_wtype_t wtype, int32_t cout, int32_t cin,
                       int32_t kh, int32_t kw, int32_t bits, squant_mode_t mode,
                       squant_output_t output, void* d_out, float* d_scales, void* stream) {
  if (!d_w || !d_out || !d_scales) return SQUANT_ERR_NULL;
  if (int rc = check_shape(cout, cin, kh, kw)) return rc;
  if (int rc = check_common(bits, (int)mode)) return rc;
  if (int rc = check_format((int)wtype, (int)output, bits, d_w, d_out)) return rc;
  const DeviceLimits lim = device_limits();
  if (!lim.ok) { (void)hipGetLastError(); return SQUANT_ERR_DEVICE; }
  const int64_t K = (int64_t)kh * kw;
  const Plan p = plan_tensor(d_w, d_out, cin, K, lim.lds_bytes);
  if (p.lds == 0) return SQUANT_ERR_UNSUPPORTED;
  Group g{p.variant, p.threads, p.lds, {}};
  g.t.push_back(TensorDesc{d_w, d_out, d_scales, cout, cin, (int32_t)K, 0});
  g.wave_members = is_k1_wave(p.variant);
  return launch_group(g, (1 << (bits - 1)) - 1, (int)mode, (int)output, (int)wtype,
                      (hipStream_t)stream);
}

int squant_quantize(const float* d_w, int32_t cout, int32_t cin, int32_t kh, int32_t kw,
                    int32_t bits, squant_mode_t mode, int8_t* d_codes, float* d_scales,
                    void* stream) {
  return squant_quantize_ex(d_w, SQUANT_W_F32, cout, cin, kh, kw, bits, mode, SQUANT_OUT_INT8,
                            d_codes, d_scales, stream);
}

size_t squant_output_bytes(int32_t cout, int32_t cin, int32_t kh, int32_t kw, squant_output_t output) {
  if (check_shape(cout, cin, kh, kw) != SQUANT_OK) return 0;
  const size_t L = (size_t)cin * kh * kw;
  switch (output) {
    case SQUANT_OUT_INT8: return (size_t)cout * L;
    case SQUANT_OUT_INT4: return (size_t)cout * ((L + 1) / 2);
    case SQUANT_OUT_F32: return (size_t)cout * L * 4;
    case SQUANT_OUT_BF16: return (size_t)cout * L * 2;
  }
  return 0;
}

// The descriptors travel in the kernel arguments and no kernel needs memory beyond its inputs
// and outputs, so no call asks for a workspace.
size_t squant_batched_workspace_bytes(int32_t) { return 0; }

int squant_quantize_batched(const squant_tensor_t* h_tensors, int32_t n_tensors, int32_t bits,
                            squant_mode_t mode, void* d_workspace, size_t workspace_bytes,
                            void* stream) {
  return squant_quantize_batched_ex(h_tensors, n_tensors, SQUANT_W_F32, bits, mode,
                                    SQUANT_OUT_INT8, d_workspace, workspace_bytes, stream);
}

int squant_quantize_batched_ex(const squant_tensor_t* h_tensors, int32_t n_tensors,
                               squant_wtype_t wtype, int32_t bits, squant_mode_t mode,
                               squant_output_t output, void* d_workspace, size_t workspace_bytes,
                               void* stream) {
  if (n_tensors < 0) return SQUANT_ERR_SHAPE;
  if (n_tensors == 0) return SQUANT_OK;
  if (!h_tensors) return SQUANT_ERR_NULL;
  if (int rc = check_common(bits, (int)mode)) return rc;
  for (int32_t i = 0; i < n_tensors; ++i) {
    const squant_tensor_t& t = h_tensors[i];
    if (!t.w || !t.codes || !t.scales) return SQUANT_ERR_NULL;
    if (int rc = check_shape(t.cout, t.cin, t.kh, t.kw)) return rc;
    if (int rc = check_format((int)wtype, (int)output, bits, t.w, t.codes)) return rc;
  }
  if (!d_workspace && workspace_bytes != 0) return SQUANT_ERR_WORKSPACE;
  const DeviceLimits lim = device_limits();
  if (!lim.ok) { (void)hipGetLastError(); return SQUANT_ERR_DEVICE; }

  // Group tensors by launch configuration.  Tensors whose variant runs in workgroups of at
  // most kMixedMaxThreads threads share ONE launch of the mixed kernel when they differ in
  // variant or launch shape (the layers of a network); a uniform set keeps its own kernel.
  std::vector<Plan> plans((size_t)n_tensors);
  const size_t lds_cap = (size_t)lim.lds_bytes - kStaticLds - sizeof(K9Shared) - sizeof(GenericShared);
  int small_kinds = 0;
  Plan small_first{};
  for (int32_t i = 0; i < n_tensors; ++i) {
    const squant_tensor_t& t = h_tensors[i];
    Plan p = plan_tensor(t.w, t.codes, t.cin, (int64_t)t.kh * t.kw, lim.lds_bytes);
    if (p.lds == 0) return SQUANT_ERR_UNSUPPORTED;
    // LDS size classes: next power of two >= 2 KB keeps the number of launches small
    size_t cls = 2048;
    while (cls < p.lds) cls <<= 1;
    p.lds = std::max(std::min(cls, lds_cap), p.lds);
    plans[(size_t)i] = p;
    if (mixable(p, lds_cap)) {
      if (small_kinds == 0) { small_first = p; small_kinds = 1; }
      else if (p.variant != small_first.variant || p.threads != small_first.threads ||
               p.lds != small_first.lds) small_kinds = 2;
    }
  }
  const bool use_mixed = small_kinds > 1;
  // Likewise the small-kernel tensors of up to kKsMixedMaxThreads threads per channel share one
  // launch when they differ in kernel size, kernels per thread or launch shape.
  int ks_kinds = 0;
  Plan ks_first{};
  for (int32_t i = 0; i < n_tensors; ++i) {
    const Plan& p = plans[(size_t)i];
    if (!is_ks(p.variant) || p.threads > kKsMixedMaxThreads) continue;
    if (ks_kinds == 0) { ks_first = p; ks_kinds = 1; }
    else if (p.variant != ks_first.variant || p.threads != ks_first.threads || p.lds != ks_first.lds) ks_kinds = 2;
  }
  const bool use_ks_mixed = ks_kinds > 1;
  // One mixed launch while its workgroups stay at 128 threads (measured: ResNet-18 set 27 %,
  // MobileNetV2 set 12 % faster than two launches, ResNet-50 set the same).  When a member
  // needs 256 threads, the channels that take one wave get a launch of one-wave workgroups of
  // their own: four times as many of them fit a compute unit.
  int widest = 0;
  for (int32_t i = 0; i < n_tensors; ++i) {
    const Plan& p = plans[(size_t)i];
    if (use_mixed && mixable(p, lds_cap) && p.variant != kGeneric) widest = std::max(widest, p.mix_threads);
  }
  const bool two_classes = widest > 2 * kWave;
  std::vector<Group> groups;
  for (int32_t i = 0; i < n_tensors; ++i) {
    const squant_tensor_t& t = h_tensors[i];
    const Plan& p = plans[(size_t)i];
    const bool in_ks_mixed = use_ks_mixed && is_ks(p.variant) && p.threads <= kKsMixedMaxThreads;
    const bool in_mixed = in_ks_mixed || (use_mixed && mixable(p, lds_cap));
    const int need_threads = in_ks_mixed ? p.threads : p.mix_threads;
    const int mixed_kind = in_ks_mixed ? kKsMixed : (two_classes && need_threads <= kWave) ? kMixedWave : kMixed;
    Group* g = nullptr;
    for (auto& c : groups) {
      if (in_mixed ? c.variant == mixed_kind
                   : (c.variant == p.variant && c.threads == p.threads && c.lds == p.lds)) { g = &c; break; }
    }
    if (!g) {
      groups.push_back(Group{in_mixed ? mixed_kind : p.variant, in_mixed ? need_threads : p.threads, p.lds, {}});
      g = &groups.back();
    }
    if (in_mixed) {
      // the workgroup size follows the specialised routines (their kernels / vectors per thread
      // depend on it); the generic routine strides by whatever size it is given, so a generic
      // member only sets the size of a launch that has no other kind of member
      if (p.variant != kGeneric) {
        g->threads = g->fixed_threads ? std::max(g->threads, need_threads) : need_threads;
        g->fixed_threads = true;
      } else if (!g->fixed_threads) {
        g->threads = std::max(g->threads, need_threads);
      }
      g->lds = std::max(g->lds, p.lds);
    }
    g->t.push_back(TensorDesc{t.w, t.codes, t.scales, t.cout, t.cin, (int32_t)((int64_t)t.kh * t.kw), 0});
    g->wave_members |= is_k1_wave(p.variant);
  }
  hipStream_t st = (hipStream_t)stream;
  const int qmax = (1 << (bits - 1)) - 1;
  for (const auto& g : groups)
    if (int rc = launch_group(g, qmax, (int)mode, (int)output, (int)wtype, st)) return rc;
  return SQUANT_OK;
}

size_t squant_activation_workspace_bytes(int32_t) { return 0; }

namespace {
// Shared by squant_activation_ranges and squant_quantize_network; every descriptor names the
// entry of d_ranges it writes.  Launches of at most kInlineBn layers each.
int launch_activation_ranges(const std::vector<BnDesc>& layers, float n_sigma, int32_t bits,
                             squant_act_range_t* d_ranges, hipStream_t st) {
  for (size_t c0 = 0; c0 < layers.size(); c0 += kInlineBn) {
    BnArgs a{};
    const int cnt = (int)std::min<size_t>(kInlineBn, layers.size() - c0);
    for (int i = 0; i < cnt; ++i) a.layer[i] = layers[c0 + i];
    a.n_sigma = n_sigma;
    a.levels_minus_1 = (int32_t)((1 << bits) - 1);
    a.out = d_ranges;
    hipLaunchKernelGGL(squant_activation_range_kernel, dim3((unsigned)cnt), dim3(256), 0, st, a);
    if (hipGetLastError() != hipSuccess) return SQUANT_ERR_DEVICE;
  }
  return SQUANT_OK;
}

int check_activation_args(int32_t bits, float n_sigma) {
  if (bits < 2 || bits > 16) return SQUANT_ERR_BITS;
  if (!(n_sigma >= 0.0f) || !(n_sigma <= 3.0e38f)) return SQUANT_ERR_SHAPE;
  return SQUANT_OK;
}
}  // namespace

int squant_activation_ranges(const squant_bn_t* h_layers, int32_t n_layers, float n_sigma,
                             int32_t bits, squant_act_range_t* d_ranges, void* d_workspace,
                             size_t workspace_bytes, void* stream) {
  if (n_layers < 0) return SQUANT_ERR_SHAPE;
  if (n_layers == 0) return SQUANT_OK;
  if (!h_layers || !d_ranges) return SQUANT_ERR_NULL;
  if (int rc = check_activation_args(bits, n_sigma)) return rc;
  std::vector<BnDesc> layers;
  layers.reserve((size_t)n_layers);
  for (int32_t i = 0; i < n_layers; ++i) {
    const squant_bn_t& l = h_layers[i];
    if (!l.gamma || !l.beta) return SQUANT_ERR_NULL;
    if (l.channels <= 0) return SQUANT_ERR_SHAPE;
    layers.push_back(BnDesc{l.gamma, l.beta, l.channels, l.relu, i, 0});
  }
  if (!d_workspace && workspace_bytes != 0) return SQUANT_ERR_WORKSPACE;
  return launch_activation_ranges(layers, n_sigma, bits, d_ranges, (hipStream_t)stream);
}

size_t squant_network_workspace_bytes(int32_t) { return 0; }

int squant_quantize_network(const squant_layer_t* h_layers, int32_t n_layers, int32_t weight_bits,
                            squant_mode_t mode, int32_t act_bits, float n_sigma,
                            squant_act_range_t* d_ranges, void* d_workspace,
                            size_t workspace_bytes, void* stream) {
  if (n_layers < 0) return SQUANT_ERR_SHAPE;
  if (n_layers == 0) return SQUANT_OK;
  if (!h_layers) return SQUANT_ERR_NULL;
  if (int rc = check_activation_args(act_bits, n_sigma)) return rc;
  std::vector<squant_tensor_t> weights((size_t)n_layers);
  std::vector<BnDesc> bns;
  for (int32_t i = 0; i < n_layers; ++i) {
    weights[(size_t)i] = h_layers[i].weight;
    const squant_bn_t& l = h_layers[i].bn;
    if (!l.gamma) continue;
    if (!l.beta || !d_ranges) return SQUANT_ERR_NULL;
    if (l.channels <= 0) return SQUANT_ERR_SHAPE;
    bns.push_back(BnDesc{l.gamma, l.beta, l.channels, l.relu, i, 0});
  }
  if (!d_workspace && workspace_bytes != 0) return SQUANT_ERR_WORKSPACE;
  if (int rc = squant_quantize_batched(weights.data(), n_layers, weight_bits, mode, nullptr, 0, stream))
    return rc;
  if (bns.empty()) return SQUANT_OK;
  return launch_activation_ranges(bns, n_sigma, act_bits, d_ranges, (hipStream_t)stream);
}

int64_t squant_max_channel_elems(int32_t kh, int32_t kw) {
  if (kh <= 0 || kw <= 0 || (int64_t)kh * kw > (1 << 20)) return 0;
  return (int64_t)1 << 30;  // the bound of the argument check: the streaming kernel takes any channel
}

const char* squant_status_string(int status) {
  switch (status) {
    case SQUANT_OK: return "ok";
    case SQUANT_ERR_NULL: return "null pointer";
    case SQUANT_ERR_SHAPE: return "bad shape";
    case SQUANT_ERR_BITS: return "bits must be in [2, 8]";
    case SQUANT_ERR_MODE: return "unknown mode";
    case SQUANT_ERR_WORKSPACE: return "workspace size given without a workspace";
    case SQUANT_ERR_DEVICE: return "HIP call failed";
    case SQUANT_ERR_UNSUPPORTED: return "unsupported (not returned by this version)";
    case SQUANT_ERR_FORMAT: return "unknown weight or output type, or misaligned buffer";
    default: return "unknown status";
  }
}

int squant_version(void) { return 200; }

}  // extern "C"
