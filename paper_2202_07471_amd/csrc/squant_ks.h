// SQuant kernel for small convolution kernels other than 3x3 (1x3, 3x1, 1x7, 7x1, 2x2, 1x5,
// 5x5 ...: K = kh*kw elements, 2 <= K <= kKsMaxK), built like the 3x3 kernel: one workgroup per
// output channel, every thread holds KPT whole kernels in registers (thread t the kernels
// t, t+G, ..., G = cin / KPT), SQuant-E, SQuant-K and the Algorithm 3 candidate are register
// arithmetic, LDS only holds the channel's biased codes for SQuant-C and the write-out.
//
// The k largest same-sign perturbations of a kernel (Algorithm 2's top-k, k <= K/2) are found
// by ranking: with unique integer keys (|p| in Q23 above an "index from the end" tie-break,
// elements of the other sign below all same-sign ones) the rank of an element is the number of
// larger keys, K(K-1)/2 comparisons in all; an element flips when its rank is below k, and the
// candidate is the element of rank k-1 (over SQuant) or k (under SQuant).
#pragma once

#include "squant_common.h"
#include "squant_io.h"
#include "squant_k9.h"  // K9Shared
#include "squant_plan.h"
#include "squant_select.h"

namespace squant {

typedef float vf2 __attribute__((ext_vector_type(2)));
// kernels start on 4-byte boundaries only
typedef vf4 vf4_dword __attribute__((aligned(4)));
typedef vf3 vf3_dword __attribute__((aligned(4)));
typedef vf2 vf2_dword __attribute__((aligned(4)));

// K consecutive floats at p (4-byte aligned) into w[K*q .. K*q+K-1], in 16-byte pieces and
// one shorter piece.
template <int K, int NW>
__device__ __forceinline__ void ks_load_kernel(float (&w)[NW], int q, const float* p) {
  const uintptr_t a = reinterpret_cast<uintptr_t>(p);
  constexpr int V4 = K / 4, R = K % 4;
#pragma unroll
  for (int j = 0; j < V4; ++j) {
    const vf4 v = *reinterpret_cast<const __attribute__((address_space(1))) vf4_dword*>(a + 16 * j);
    w[K * q + 4 * j] = v.x; w[K * q + 4 * j + 1] = v.y; w[K * q + 4 * j + 2] = v.z; w[K * q + 4 * j + 3] = v.w;
  }
  if (R == 3) {
    const vf3 v = *reinterpret_cast<const __attribute__((address_space(1))) vf3_dword*>(a + 16 * V4);
    w[K * q + 4 * V4] = v.x; w[K * q + 4 * V4 + 1] = v.y; w[K * q + 4 * V4 + 2] = v.z;
  } else if (R == 2) {
    const vf2 v = *reinterpret_cast<const __attribute__((address_space(1))) vf2_dword*>(a + 16 * V4);
    w[K * q + 4 * V4] = v.x; w[K * q + 4 * V4 + 1] = v.y;
  } else if (R == 1) {
    w[K * q + 4 * V4] = *reinterpret_cast<const __attribute__((address_space(1))) float*>(a + 16 * V4);
  }
}

// SQuant-E, SQuant-K and the candidate update for one K-element kernel held in registers
// (straight-line code, as for 3x3).  Arguments as for k9_solve.
template <int K, int NW, bool FAST, int MODE>
__device__ __forceinline__ void ks_solve(const float (&w)[NW], int q, float s, float rs, float qmaxf,
                                         float (&cf)[K], int32_t& esum, uint32_t& cand_w,
                                         int& cand_i, uint32_t& zero) {
  constexpr int IB = K <= 16 ? 4 : K <= 32 ? 5 : 6;  // bits of the index tie-break
  constexpr int IM = (1 << IB) - 1;
  const int W0 = K * q;
  float c[K];
  int32_t P[K];
#pragma unroll
  for (int i = 0; i < K; ++i) {
    const float x = FAST ? div_by_reciprocal(w[W0 + i], s, rs) : w[W0 + i] / s;
    const float xc = __builtin_amdgcn_fmed3f(x, -qmaxf, qmaxf);
    c[i] = rintf(xc);
    const float p = c[i] - xc;  // exact
    // Q23 through the low mantissa bits of p * 2^23 + 1.5 * 2^23 (one rounding, half to even)
    P[i] = __float_as_int(__builtin_fmaf(p, 8388608.0f, 12582912.0f)) - 0x4B400000;
  }
  cand_w = kNoCandidate;
  cand_i = 0;
  if (MODE == SQUANT_MODE_E) {
#pragma unroll
    for (int i = 0; i < K; ++i) cf[i] = c[i] + 128.0f;
    return;
  }

  // ---- SQuant-K (Algorithm 2 on one kernel) ----
  int32_t E = 0;
#pragma unroll
  for (int i = 0; i < K; ++i) E += P[i];
  const int32_t smask = E >> 31;
  const int32_t A = (E ^ smask) - smask;
  const int32_t k = (MODE == SQUANT_MODE_EC) ? 0 : (int32_t)((uint32_t)(A + kHalf - 1) >> 23);
  const int32_t r = A - (k << 23);  // |sum| left after k flips, < 0: over SQuant
  esum += (r ^ smask) - smask;
  zero |= (E == 0 ? 1u : 0u) << q;

  // unique keys: 2^IB |p| + (IM - i) >= 2^IB for the elements with the sign of the sum, below
  // 2^IB for all others; |P| <= 2^22 fits the 24-bit multiply
  int32_t key[K], rank[K];
#pragma unroll
  for (int i = 0; i < K; ++i) {
    key[i] = __mul24(P[i], smask ? -(1 << IB) : (1 << IB)) + (IM - i);
    rank[i] = i;  // rank = #{larger keys}: i counts the pairs (j < i), corrected below
  }
#pragma unroll
  for (int i = 0; i < K; ++i)
#pragma unroll
    for (int j = i + 1; j < K; ++j) {
      const int32_t gt = key[j] > key[i] ? 1 : 0;
      rank[i] += gt;
      rank[j] -= gt;
    }

  // flip the k largest: code -= sign(E)
  const float flip = smask ? 129.0f : 127.0f;
#pragma unroll
  for (int i = 0; i < K; ++i) cf[i] = c[i] + (rank[i] < k ? flip : 128.0f);
  if (MODE == SQUANT_MODE_EK) return;

  // ---- perturbation update (Algorithm 3): the kernel's candidate for SQuant-C ----
  const bool over = r < 0;
  const int32_t want = over ? k - 1 : k;  // over: last flipped; under: first un-flipped (k <= K/2 < K)
  int32_t ck = 0;
#pragma unroll
  for (int i = 0; i < K; ++i) ck |= rank[i] == want ? key[i] : 0;
  const uint32_t mag = (uint32_t)ck >> IB;  // |p| of that element before any flip (if same-sign)
  const uint32_t absv = over ? (uint32_t)kOne - mag : mag;
  const uint32_t neg = (over ? ~(uint32_t)smask : (uint32_t)smask) & (1u << 23);
  cand_w = ck >= (1 << IB) ? (absv | neg) : kNoCandidate;
  cand_i = IM - (ck & IM);
}

// Cold path: the SQuant-C candidate of a kernel whose perturbation sum is exactly zero (nothing
// masked: the largest |p| of either sign, lowest index first), recomputed from memory.
__device__ __noinline__ int2 ks_zero_sum_candidate(const void* w, size_t first, int K, int wtype,
                                                   float s, float qmaxf) {
  int32_t best = 0, bv = 0;
  int bi = 0;
  for (int i = 0; i < K; ++i) {
    float x = load_weight(w, first + i, wtype) / s;
    x = fminf(fmaxf(x, -qmaxf), qmaxf);
    const float p = rintf(x) - x;
    const int32_t P = __float2int_rn(p * 8388608.0f);
    const int32_t ap = P < 0 ? -P : P;
    if (ap > best) { best = ap; bv = P; bi = i; }
  }
  return make_int2(bv, bi);
}

template <int K, int KPT, bool FAST, int MODE>
__device__ __forceinline__ void ks_solve_all(const float (&w)[K * KPT], float s, float rs, float qmaxf,
                                             uint8_t* code8, int t, int G, int32_t& esum,
                                             uint32_t (&cv)[KPT], int (&ci)[KPT], uint32_t& zero) {
#pragma unroll
  for (int q = 0; q < KPT; ++q) {
    float cf[K];
    ks_solve<K, K * KPT, FAST, MODE>(w, q, s, rs, qmaxf, cf, esum, cv[q], ci[q], zero);
    const int n = t + q * G;
#pragma unroll
    for (int i = 0; i < K; ++i) code8[K * n + i] = (uint8_t)(int)cf[i];
  }
}

// One workgroup per output channel of N = KPT * G kernels, N * K a multiple of 4.
template <int MODE, int K, int KPT>
__device__ __forceinline__ void ks_channel(const LaunchArgs& a, const TensorDesc& d, int m,
                                           unsigned char* smem, K9Shared& sh) {
  constexpr bool kChannelStage = MODE == SQUANT_MODE_EKC || MODE == SQUANT_MODE_EC;
  const int T = blockDim.x, tid = threadIdx.x;
  const float qmaxf = (float)a.qmax;
  uint8_t* code8 = reinterpret_cast<uint8_t*>(smem);  // biased codes: code + 128

  const int N = d.N, G = N / KPT;
  const int L = K * N, nvec = L >> 2;
  const bool active = tid < G;
  const int t = active ? tid : 0;  // idle threads shadow thread 0's loads and write nothing
  float w[K * KPT];
  if (a.wtype == SQUANT_W_F32) {
    const float* src = static_cast<const float*>(d.w) + (size_t)m * L;
#pragma unroll
    for (int q = 0; q < KPT; ++q) ks_load_kernel<K>(w, q, src + (size_t)K * (size_t)(t + q * G));
  } else {
    const size_t first = (size_t)m * L;
#pragma unroll
    for (int q = 0; q < KPT; ++q)
#pragma unroll
      for (int i = 0; i < K; ++i)
        w[K * q + i] = load_weight(d.w, first + (size_t)K * (size_t)(t + q * G) + i, a.wtype);
  }
  if (kChannelStage) select_reset(sh.sel);  // before the first barrier

  float amax = 0.0f;
#pragma unroll
  for (int j = 0; j < K * KPT; ++j) amax = fmaxf(amax, fabsf(w[j]));
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
      ks_solve_all<K, KPT, true, MODE>(w, s, 1.0f / s, qmaxf, code8, t, G, esum, cv, ci, zero);
    } else {
      ks_solve_all<K, KPT, false, MODE>(w, s, 0.0f, qmaxf, code8, t, G, esum, cv, ci, zero);
    }
    if (kChannelStage && zero != 0) {
#pragma unroll
      for (int q = 0; q < KPT; ++q)
        if (zero & (1u << q)) {
          const int2 z = ks_zero_sum_candidate(d.w, (size_t)m * L + (size_t)K * (size_t)(t + q * G), K,
                                               a.wtype, s, qmaxf);
          cv[q] = candidate_word(z.x);
          ci[q] = z.y;
        }
    }
  }
  if (kChannelStage) {
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
      for (int q = 0; q < KPT; ++q) { cn[q] = t + q * G; cpos[q] = K * cn[q] + ci[q]; }
      channel_stage<KPT, 1>(cv, cpos, cn, sgn, (uint32_t)(kc > N ? N : kc),
                            reinterpret_cast<uint32_t*>(smem), sh.sel);
    }
  }
  __syncthreads();

  emit_channel(reinterpret_cast<const uint32_t*>(smem), nvec, d.out, m, s, a.out_format, tid, T);
}

// Up to 256 threads: compiled for five waves per SIMD (measured 1-3.5 % faster than the
// compiler's own choice of four for 1x3, 1x7 and 2x2 kernels; six costs 5x5 27 %, eight spills).
template <int MAX_THREADS, int MODE, int K, int KPT>
__global__ void __launch_bounds__(MAX_THREADS)
    __attribute__((amdgpu_waves_per_eu(MAX_THREADS > 256 ? 1 : 5))) squant_channel_ks(LaunchArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];  // K*N bytes of codes
  __shared__ K9Shared sh;
  int m;
  const TensorDesc d = locate(a, blockIdx.x, m);
  ks_channel<MODE, K, KPT>(a, d, m, smem, sh);
}

// One launch for tensors of different small-kernel shapes (the factorised 1x7 / 7x1 / 1x3 / 3x1
// and 5x5 layers of a network): every workgroup looks up its tensor and takes the routine for
// its kernel size and kernels per thread.  The workgroup may be larger than a member needs;
// its extra threads idle.
// Compiled for four waves per SIMD (the 5x5 routine alone would take 130 VGPRs and leave three;
// measured 3 % faster on the InceptionV3-style set, five and six waves are no better).
template <int MODE>
__global__ void __launch_bounds__(256)
    __attribute__((amdgpu_waves_per_eu(4))) squant_channel_ks_mixed(LaunchArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ K9Shared sh;
  int m;
  const TensorDesc d = locate(a, blockIdx.x, m);
  switch (4 * d.K + ks_kpt_log2(d.N, d.K)) {
#define SQ_KS_CASE(K, LG) \
    case 4 * K + LG: ks_channel<MODE, K, (1 << LG)>(a, d, m, smem, sh); break;
    SQ_KS_CASE(2, 0) SQ_KS_CASE(2, 1) SQ_KS_CASE(2, 2) SQ_KS_CASE(2, 3)
    SQ_KS_CASE(3, 0) SQ_KS_CASE(3, 1) SQ_KS_CASE(3, 2) SQ_KS_CASE(3, 3)
    SQ_KS_CASE(4, 0) SQ_KS_CASE(4, 1) SQ_KS_CASE(4, 2) SQ_KS_CASE(4, 3)
    SQ_KS_CASE(5, 0) SQ_KS_CASE(5, 1) SQ_KS_CASE(5, 2)
    SQ_KS_CASE(7, 0) SQ_KS_CASE(7, 1) SQ_KS_CASE(7, 2)
    SQ_KS_CASE(25, 0)
#undef SQ_KS_CASE
    default: break;  // the host puts no other tensor into this launch
  }
}

}  // namespace squant
