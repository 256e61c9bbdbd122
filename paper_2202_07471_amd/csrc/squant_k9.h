// SQuant kernel for 3x3 convolutions (K = kh*kw = 9), the bulk of a CNN's weights.
//
// One workgroup per output channel, one thread per FOUR 3x3 kernels.  Nothing is staged:
// thread t reads kernels t, t+G, t+2G, t+3G (G = cin/4) straight from HBM as three 12-byte
// vectors each, so neighbouring lanes read neighbouring kernels and the three loads of a
// wave cover one contiguous 2304-byte span.  From there SQuant-E, SQuant-K and the
// Algorithm 3 candidate are pure register arithmetic: the k <= 4 largest same-sign
// perturbations of a kernel come out of a 25-operation three-input (max3/med3/min3) selection network on unique integer
// keys (|p| in Q23 above a 4-bit "15 - index" tie-break).  LDS only holds the channel's
// int8 codes, for the channel-wise flips of SQuant-C (run once per channel on the 4
// candidates each thread holds) and for a coalesced 16-byte write-out; occupancy is left
// to the register file.
#pragma once

#include "squant_common.h"
#include "squant_io.h"
#include "squant_select.h"

namespace squant {

struct alignas(16) K9Shared {
  float red_f[16];
  int64_t red_i[16];
  SelectShared sel;
};

// SQuant-E, SQuant-K and the candidate update for one 3x3 kernel held in registers.
// Straight-line code on purpose: the four kernels of a thread are scheduled as one region,
// and a branch between them was measured to cost 20%.
//   w, q    the kernel's nine weights are w[9q .. 9q+8]
//   FAST    take the quotients through the reciprocal rs = 1/s
//   MODE    SQUANT_MODE_*
//   cf      out: the final codes as floats, biased by +128
//   esum    += the kernel's Q23 perturbation sum after SQuant-K
//   cand_w  the kernel's SQuant-C candidate as a candidate word (squant_select.h)
//   cand_i  its element index 0..8
//   zero    |= 1 << Q when the kernel's perturbation sum is exactly 0 (its candidate is then
//           worked out separately, see k9_zero_sum_candidate)
template <int NW, bool FAST, int MODE>
__device__ __forceinline__ void k9_solve(const float (&w)[NW], int q, float s, float rs, float qmaxf,
                                         float (&cf)[9], int32_t& esum, uint32_t& cand_w,
                                         int& cand_i, uint32_t& zero) {
  const int W0 = 9 * q;  // a constant once the caller's loop over q is unrolled
  float c[9];
  int32_t P[9];
#pragma unroll
  for (int i = 0; i < 9; ++i) {
    // x = w / s: either way the IEEE binary32 quotient
    const float x = FAST ? div_by_reciprocal(w[W0 + i], s, rs) : w[W0 + i] / s;
    const float xc = __builtin_amdgcn_fmed3f(x, -qmaxf, qmaxf);
    c[i] = rintf(xc);
    const float p = c[i] - xc;  // exact
    // Q23: p * 2^23 + 1.5 * 2^23 lies in [2^23, 2^24], where a float is an integer, so the one
    // rounding of the FMA is the round-half-even of p * 2^23 and the integer sits in the
    // low mantissa bits
    P[i] = __float_as_int(__builtin_fmaf(p, 8388608.0f, 12582912.0f)) - 0x4B400000;
  }
  cand_w = kNoCandidate;
  cand_i = 0;
  if (MODE == SQUANT_MODE_E) {
#pragma unroll
    for (int i = 0; i < 9; ++i) cf[i] = c[i] + 128.0f;
    return;
  }

  // ---- SQuant-K (Algorithm 2 on one kernel) ----
  int32_t E = 0;
#pragma unroll
  for (int i = 0; i < 9; ++i) E += P[i];
  const int32_t smask = E >> 31;                 // all ones when the sum is negative
  const int32_t A = (E ^ smask) - smask;         // |E|
  const int32_t k = (MODE == SQUANT_MODE_EC) ? 0 : (int32_t)((uint32_t)(A + kHalf - 1) >> 23);
  const int32_t r = A - (k << 23);               // |sum| left after k flips, < 0: over SQuant
  esum += (r ^ smask) - smask;
  zero |= (E == 0 ? 1u : 0u) << q;

  // unique keys: 16 |p| + (15 - i) >= 16 for the elements with the sign of the sum, < 16 for
  // all others; |P| <= 2^22 fits the 24-bit multiply-add
  int32_t key[9], srt[5];
#pragma unroll
  for (int i = 0; i < 9; ++i) key[i] = __mul24(P[i], smask ? -16 : 16) + (15 - i);
  top5_of_9(key, srt);
  int32_t s_km1 = 0x7fffffff, s_k = srt[0];      // (k-th, (k+1)-th) largest key, 1-based
  if (k >= 1) { s_km1 = srt[0]; s_k = srt[1]; }
  if (k >= 2) { s_km1 = srt[1]; s_k = srt[2]; }
  if (k >= 3) { s_km1 = srt[2]; s_k = srt[3]; }
  if (k >= 4) { s_km1 = srt[3]; s_k = srt[4]; }

  // flip the k largest: code -= sign(E)
  const float flip = smask ? 129.0f : 127.0f;
#pragma unroll
  for (int i = 0; i < 9; ++i) cf[i] = c[i] + (key[i] >= s_km1 ? flip : 128.0f);
  if (MODE == SQUANT_MODE_EK) return;

  // ---- perturbation update (Algorithm 3): the kernel's candidate for SQuant-C ----
  const bool over = r < 0;
  const int32_t ck = over ? s_km1 : s_k;         // over: last flipped; under: first un-flipped
  const uint32_t mag = (uint32_t)ck >> 4;        // |p| of that element before any flip
  // over: the post-flip value kOne - mag with the sign opposite to the sum; under: mag with
  // the sign of the sum
  const uint32_t absv = over ? (uint32_t)kOne - mag : mag;
  const uint32_t neg = (over ? ~(uint32_t)smask : (uint32_t)smask) & (1u << 23);
  cand_w = ck >= 16 ? (absv | neg) : kNoCandidate;
  cand_i = 15 - (ck & 15);
}

// Cold path: the SQuant-C candidate of a kernel whose perturbation sum is exactly zero
// (nothing is masked then: the largest |p| of either sign, lowest index first).  Such a
// kernel has k = 0, so its perturbations are those of plain rounding and are recomputed
// here from the weights in memory.
__device__ __noinline__ int2 k9_zero_sum_candidate(const void* w, size_t first, int wtype, float s,
                                                   float qmaxf) {
  int32_t best = 0, bv = 0;
  int bi = 0;
  for (int i = 0; i < 9; ++i) {
    float x = load_weight(w, first + i, wtype) / s;
    x = fminf(fmaxf(x, -qmaxf), qmaxf);
    const float p = rintf(x) - x;
    const int32_t P = __float2int_rn(p * 8388608.0f);
    const int32_t ap = P < 0 ? -P : P;
    if (ap > best) { best = ap; bv = P; bi = i; }
  }
  return make_int2(bv, bi);  // (candidate perturbation, element index)
}

// Kernel q of a thread: nine floats at `base` (uniform, the channel's kernels q*G ...)
// plus the lane's element offset, as three 12-byte loads, into w[9q .. 9q+8].
template <int NW>
__device__ __forceinline__ void k9_load_kernel(float (&w)[NW], int q, const float* base,
                                               uint32_t lane_off) {
#pragma unroll
  for (int j = 0; j < 3; ++j) {
    const vf3 v = load_global_f3(base + (lane_off + 3 * j));
    w[9 * q + 3 * j] = v.x; w[9 * q + 3 * j + 1] = v.y; w[9 * q + 3 * j + 2] = v.z;
  }
}

// The same for 16-bit weights (binary16 or bfloat16).  Kernel n starts at half-word 9n of
// the channel, which is dword aligned for even n only, so five aligned dwords starting at
// half-word 9n - (n & 1) are read and shifted down by one half-word for odd n.  chan32 is the
// channel's first dword (the channel has 9 * cin half-words, cin % 4 == 0, so it is dword
// aligned and ends with the last kernel's last half-word: no load reaches past it).
template <int NW>
__device__ __forceinline__ void k9_load_kernel16(float (&w)[NW], int q, const uint32_t* chan32,
                                                 uint32_t n, bool bf16) {
  const uint32_t h0 = 9u * n;
  const uint32_t sh = (h0 & 1u) << 4;
  const uint32_t* p = chan32 + (h0 >> 1);
  uint32_t d[5];
#pragma unroll
  for (int j = 0; j < 5; ++j) d[j] = load_global_u1(p + j);
  uint32_t u[5];
#pragma unroll
  for (int j = 0; j < 4; ++j) u[j] = __builtin_amdgcn_alignbit(d[j + 1], d[j], sh);
  u[4] = d[4] >> sh;
#pragma unroll
  for (int j = 0; j < 4; ++j) widen_pair(u[j], bf16, w[9 * q + 2 * j], w[9 * q + 2 * j + 1]);
  float unused;
  widen_pair(u[4], bf16, w[9 * q + 8], unused);
}

template <int KPT, bool FAST, int MODE>
__device__ __forceinline__ void k9_solve_all(const float (&w)[9 * KPT], float s, float rs, float qmaxf,
                                             uint8_t* code8, int t, int G, int32_t& esum,
                                             uint32_t (&cv)[KPT], int (&ci)[KPT], uint32_t& zero) {
#pragma unroll
  for (int q = 0; q < KPT; ++q) {
    float cf[9];
    k9_solve<9 * KPT, FAST, MODE>(w, q, s, rs, qmaxf, cf, esum, cv[q], ci[q], zero);
    const int n = t + q * G;
#pragma unroll
    for (int i = 0; i < 9; ++i) code8[9 * n + i] = (uint8_t)(int)cf[i];
  }
}

// One workgroup per output channel.  Thread t owns the KPT 3x3 kernels t, t + G, t + 2G, ...
// (G = cin / KPT); KPT is 4 for wide layers and 2 or 1 for narrow ones, so that the waves
// stay full.
template <int MODE, int KPT>
__device__ __forceinline__ void k9_channel(const LaunchArgs& a, const TensorDesc& d, int m,
                                           unsigned char* smem, K9Shared& sh) {
  constexpr bool kChannelStage = MODE == SQUANT_MODE_EKC || MODE == SQUANT_MODE_EC;
  const int T = blockDim.x, tid = threadIdx.x;
  const float qmaxf = (float)a.qmax;
  uint8_t* code8 = reinterpret_cast<uint8_t*>(smem);  // biased codes: code + 128

  const int N = d.N, G = N / KPT;
  const int L = 9 * N, nvec = L >> 2;  // dwords of codes (cin % 4 == 0)
  const bool active = tid < G;
  const int t = active ? tid : 0;  // idle threads shadow thread 0's loads and write nothing
  float w[9 * KPT];
  if (a.wtype == SQUANT_W_F32) {
    const float* src = static_cast<const float*>(d.w) + (size_t)m * L;
#pragma unroll
    for (int q = 0; q < KPT; ++q) k9_load_kernel(w, q, src + (size_t)q * (9 * G), 9u * (uint32_t)t);
  } else {
    const uint32_t* chan32 =
        reinterpret_cast<const uint32_t*>(static_cast<const uint16_t*>(d.w) + (size_t)m * L);
    const bool bf16 = a.wtype == SQUANT_W_BF16;
#pragma unroll
    for (int q = 0; q < KPT; ++q) k9_load_kernel16(w, q, chan32, (uint32_t)(t + q * G), bf16);
  }
  if (kChannelStage) select_reset(sh.sel);  // before the first barrier

  float amax = 0.0f;
#pragma unroll
  for (int j = 0; j + 1 < 9 * KPT; j += 2) amax = fmaxf(fmaxf(amax, fabsf(w[j])), fabsf(w[j + 1]));
  if ((9 * KPT) & 1) amax = fmaxf(amax, fabsf(w[9 * KPT - 1]));
  amax = block_max_dpp1(amax, sh.red_f);
  const float s = amax > 0.0f ? amax / qmaxf : 1.0f;
  if (tid == 0) d.scales[m] = s;

  int32_t esum = 0;
  uint32_t cv[KPT];
  int ci[KPT];
#pragma unroll
  for (int q = 0; q < KPT; ++q) { cv[q] = kNoCandidate; ci[q] = 0; }
  uint32_t zero = 0;
  if (active) {
    if (amax >= 0x1p-60f && amax <= 0x1p60f) {  // uniform over the workgroup
      k9_solve_all<KPT, true, MODE>(w, s, 1.0f / s, qmaxf, code8, t, G, esum, cv, ci, zero);
    } else {
      k9_solve_all<KPT, false, MODE>(w, s, 0.0f, qmaxf, code8, t, G, esum, cv, ci, zero);
    }
    if (kChannelStage && zero != 0) {
#pragma unroll
      for (int q = 0; q < KPT; ++q)
        if (zero & (1u << q)) {
          const int2 z = k9_zero_sum_candidate(d.w, (size_t)m * L + 9 * (t + q * G), a.wtype, s, qmaxf);
          cv[q] = candidate_word(z.x);
          ci[q] = z.y;
        }
    }
  }
  if (kChannelStage) {
    // candidates into the histogram before the wanted sign is known: one barrier then
    // publishes the codes, the partial sums and the histogram
    if (active) {
#pragma unroll
      for (int q = 0; q < KPT; ++q) count_candidate(sh.sel, cv[q]);
    }
    const int64_t ec = block_sum_dpp1(esum, sh.red_i);
    const int sgn = sign_of(ec);
    const int64_t kc = flips_for(ec < 0 ? -ec : ec);
    if (kc > 0) {
      int cpos[KPT], cn[KPT];
#pragma unroll
      for (int q = 0; q < KPT; ++q) { cn[q] = t + q * G; cpos[q] = 9 * cn[q] + ci[q]; }
      channel_stage<KPT, 1>(cv, cpos, cn, sgn, (uint32_t)(kc > N ? N : kc),
                            reinterpret_cast<uint32_t*>(smem), sh.sel);
    }
  }
  __syncthreads();

  emit_channel(reinterpret_cast<const uint32_t*>(smem), nvec, d.out, m, s, a.out_format, tid, T);
}

template <int MAX_THREADS, int MODE, int KPT>
__global__ void __launch_bounds__(MAX_THREADS) squant_channel_k9(LaunchArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];  // 9*N bytes of codes
  __shared__ K9Shared sh;
  int m;
  const TensorDesc d = locate(a, blockIdx.x, m);
  k9_channel<MODE, KPT>(a, d, m, smem, sh);
}

// ---------------------------------------------------------------------------
// Depthwise 3x3 convolutions (cin per group = 1): an output channel is a single 3x3 kernel,
// so one thread takes a whole channel - its own absmax scale, SQuant-E and SQuant-K in
// registers through k9_solve.  SQuant-C on a one-kernel channel: after SQuant-K the
// channel's sum is the kernel's, at most 0.5, so nothing flips (E&K&C equals E&K); without
// SQuant-K (mode E&C) the kernel's one candidate flips when the sum rounds to 1 or more.
// `item` is the workgroup's index within the tensor: thread t has channel item * T + t.
// No workgroup-wide step, no LDS.
// ---------------------------------------------------------------------------
template <int MODE>
__device__ __forceinline__ void dw9_channels(const LaunchArgs& a, const TensorDesc& d, int item) {
  constexpr int KM = MODE == SQUANT_MODE_EKC ? SQUANT_MODE_EK : MODE;
  const int c = item * (int)blockDim.x + (int)threadIdx.x;
  if (c >= d.M) return;
  const float qmaxf = (float)a.qmax;
  float w[9];
  if (a.wtype == SQUANT_W_F32) {
    k9_load_kernel(w, 0, static_cast<const float*>(d.w), 9u * (uint32_t)c);
  } else {
#pragma unroll
    for (int i = 0; i < 9; ++i) w[i] = load_weight(d.w, 9 * (size_t)c + i, a.wtype);
  }
  float amax = 0.0f;
#pragma unroll
  for (int i = 0; i < 9; ++i) amax = fmaxf(amax, fabsf(w[i]));
  const float s = amax > 0.0f ? amax / qmaxf : 1.0f;
  d.scales[c] = s;

  float cf[9];
  int32_t esum = 0;
  uint32_t cw = kNoCandidate, zero = 0;
  int ci = 0;
  k9_solve<9, false, KM>(w, 0, s, 0.0f, qmaxf, cf, esum, cw, ci, zero);
  if (MODE == SQUANT_MODE_EC) {
    const int32_t mag = esum < 0 ? -esum : esum;
    if (flips_for(mag) >= 1 && cw != kNoCandidate) {
      const float step = esum > 0 ? -1.0f : 1.0f;  // one step against the sum
#pragma unroll
      for (int i = 0; i < 9; ++i) cf[i] += (i == ci) ? step : 0.0f;
    }
  }

  int code[9];
#pragma unroll
  for (int i = 0; i < 9; ++i) code[i] = (int)cf[i] - 128;
  if (a.out_format == SQUANT_OUT_INT8) {
    int8_t* out = static_cast<int8_t*>(d.out) + 9 * (size_t)c;
#pragma unroll
    for (int i = 0; i < 9; ++i) out[i] = (int8_t)code[i];
  } else if (a.out_format == SQUANT_OUT_INT4) {
    uint8_t* out = static_cast<uint8_t*>(d.out) + 5 * (size_t)c;  // rows of (9 + 1) / 2 bytes
#pragma unroll
    for (int j = 0; j < 5; ++j) {
      const uint32_t lo = (uint32_t)code[2 * j] & 0xFu;
      const uint32_t hi = j < 4 ? ((uint32_t)code[2 * j + 1] & 0xFu) : 0u;
      out[j] = (uint8_t)(lo | (hi << 4));
    }
  } else if (a.out_format == SQUANT_OUT_BF16) {
    uint16_t* out = static_cast<uint16_t*>(d.out) + 9 * (size_t)c;
#pragma unroll
    for (int i = 0; i < 9; ++i) out[i] = (uint16_t)bf16_bits((float)code[i] * s);
  } else {  // SQUANT_OUT_F32
    float* out = static_cast<float*>(d.out) + 9 * (size_t)c;
#pragma unroll
    for (int i = 0; i < 9; ++i) out[i] = (float)code[i] * s;
  }
}

template <int MODE>
__global__ void __launch_bounds__(256) squant_channel_dw9(LaunchArgs a) {
  int m;
  const TensorDesc d = locate(a, blockIdx.x, m);
  dw9_channels<MODE>(a, d, m);
}

}  // namespace squant
