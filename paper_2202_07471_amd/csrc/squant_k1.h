// SQuant kernel for 1x1 convolutions and fully connected layers (K = kh*kw = 1).
//
// With one element per kernel SQuant-K has nothing to do (k = round(|p|) = 0 for |p| <= 0.5,
// Section 3.4), every element is its own kernel, and its rounding perturbation is its
// SQuant-C candidate (Algorithm 3, "under SQuant" with k = 0).  One workgroup per output
// channel; a thread takes NV 16-byte vectors of the channel, vector j of thread t being
// vector t + j*T, so every load instruction of a wave reads 1 KB of consecutive weights.
// SQuant-E runs in registers, the int8 codes go to LDS four to a dword, and SQuant-C is the
// same LDS radix select as for the 3x3 kernel, over all cin elements of the channel.
#pragma once

#include "squant_common.h"
#include "squant_io.h"
#include "squant_k9.h"  // K9Shared
#include "squant_select.h"

namespace squant {

__device__ __forceinline__ vf4 load_global_f4_stream(const float* p) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_nontemporal_load(
      reinterpret_cast<const __attribute__((address_space(1))) vf4*>(reinterpret_cast<uintptr_t>(p)));
#else
  return *reinterpret_cast<const vf4*>(p);
#endif
}

template <int MODE, int NV>
__device__ __forceinline__ void k1_channel(const LaunchArgs& a, const TensorDesc& d, int m,
                                           unsigned char* smem, K9Shared& sh) {
  constexpr bool kChannelStage = MODE == SQUANT_MODE_EKC || MODE == SQUANT_MODE_EC;
  constexpr int NE = 4 * NV;  // elements per thread
  const int T = blockDim.x, tid = threadIdx.x;
  const float qmaxf = (float)a.qmax;
  uint32_t* code32 = reinterpret_cast<uint32_t*>(smem);

  const int N = d.N, nvec = N >> 2;  // cin % 4 == 0
  float w[NE];
  if (a.wtype == SQUANT_W_F32) {
    const float* src = static_cast<const float*>(d.w) + (size_t)m * N;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int idx = tid + j * T;
      vf4 v = {0.0f, 0.0f, 0.0f, 0.0f};
      if (idx < nvec) v = load_global_f4_stream(src + 4 * idx);
      w[4 * j] = v.x; w[4 * j + 1] = v.y; w[4 * j + 2] = v.z; w[4 * j + 3] = v.w;
    }
  } else {  // 16-bit weights: the same four elements per vector, 8 bytes
    const uint16_t* src = static_cast<const uint16_t*>(d.w) + (size_t)m * N;
    const bool bf16 = a.wtype == SQUANT_W_BF16;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int idx = tid + j * T;
      vu2 v = {0u, 0u};
      if (idx < nvec) v = load_global_u2_stream(src + 4 * idx);
      widen_pair(v.x, bf16, w[4 * j], w[4 * j + 1]);
      widen_pair(v.y, bf16, w[4 * j + 2], w[4 * j + 3]);
    }
  }
  if (kChannelStage) select_reset(sh.sel);  // before the first barrier

  float amax = 0.0f;
#pragma unroll
  for (int e = 0; e < NE; e += 2) amax = fmaxf(fmaxf(amax, fabsf(w[e])), fabsf(w[e + 1]));
  amax = block_max_dpp1(amax, sh.red_f);
  const float s = amax > 0.0f ? amax / qmaxf : 1.0f;
  if (tid == 0) d.scales[m] = s;
  const bool fast = amax >= 0x1p-60f && amax <= 0x1p60f;  // uniform over the workgroup
  const float rs = 1.0f / s;

  // ---- SQuant-E (Algorithm 1): code, and the element's perturbation as candidate word ----
  int32_t esum = 0;
  uint32_t cw[NE];
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    uint32_t packed = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float wv = w[4 * j + e];
      const float x = fast ? div_by_reciprocal(wv, s, rs) : wv / s;  // the IEEE quotient either way
      const float xc = __builtin_amdgcn_fmed3f(x, -qmaxf, qmaxf);
      const float c = rintf(xc);
      packed = __builtin_amdgcn_cvt_pk_u8_f32(c + 128.0f, e, packed);
      if (kChannelStage) {
        const float p = c - xc;  // exact
        const int32_t P = __float_as_int(__builtin_fmaf(p, 8388608.0f, 12582912.0f)) - 0x4B400000;
        esum += P;
        cw[4 * j + e] = candidate_word(P);
      }
    }
    const int idx = tid + j * T;
    if (idx < nvec) code32[idx] = packed;
  }

  if (kChannelStage) {
#pragma unroll
    for (int j = 0; j < NV; ++j)
      if (tid + j * T < nvec) {
#pragma unroll
        for (int e = 0; e < 4; ++e) count_candidate(sh.sel, cw[4 * j + e]);
      }
    const int64_t ec = block_sum_dpp1(esum, sh.red_i);  // its barrier publishes codes and histogram
    const int sgn = sign_of(ec);
    const int64_t kc = flips_for(ec < 0 ? -ec : ec);
    if (kc > 0) {
      int pos[NE];
#pragma unroll
      for (int j = 0; j < NV; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          pos[4 * j + e] = 4 * (tid + j * T) + e;
          if (tid + j * T >= nvec) cw[4 * j + e] = kNoCandidate;
        }
      channel_stage<NE, 4>(cw, pos, pos, sgn, (uint32_t)(kc > N ? N : kc), code32, sh.sel);
    }
  }
  __syncthreads();

  emit_channel(code32, nvec, d.out, m, s, a.out_format, tid, T);
}

template <int MAX_THREADS, int MODE, int NV>
__global__ void __launch_bounds__(MAX_THREADS) squant_channel_k1(LaunchArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];  // N bytes of biased codes
  __shared__ K9Shared sh;
  int m;
  const TensorDesc d = locate(a, blockIdx.x, m);
  k1_channel<MODE, NV>(a, d, m, smem, sh);
}

}  // namespace squant
