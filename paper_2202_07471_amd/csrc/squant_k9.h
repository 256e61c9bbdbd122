// SQuant kernel for 3x3 convolutions (K = kh*kw = 9), the bulk of a CNN's weights.
//
// One workgroup per output channel, one thread per FOUR consecutive 3x3 kernels:
// 36 floats = nine 16-byte vectors in, 36 int8 = nine dwords out, so every LDS
// access of a thread is a full aligned vector.  The channel is streamed from HBM
// into LDS with fully coalesced 16-byte loads, each thread pulls its 36 weights
// into registers, and from there SQuant-E, SQuant-K and the Algorithm 3 candidate
// are pure register arithmetic: the k <= 4 largest same-sign perturbations of a
// kernel come out of a 22-exchange selection network on unique integer keys
// (|p| in Q24 above a 4-bit "15 - index" tie-break).  SQuant-C then runs once per
// channel on the 4 candidates each thread holds.
#pragma once

#include "squant_common.h"
#include "squant_select.h"

namespace squant {

typedef float vf4 __attribute__((ext_vector_type(4)));
typedef uint32_t vu4 __attribute__((ext_vector_type(4)));

// 16-byte load / store through the global (not flat) address space
__device__ __forceinline__ vf4 load_global_f4(const float* p) {
#if defined(__HIP_DEVICE_COMPILE__)
  return *reinterpret_cast<const __attribute__((address_space(1))) vf4*>(reinterpret_cast<uintptr_t>(p));
#else
  return *reinterpret_cast<const vf4*>(p);
#endif
}
__device__ __forceinline__ void store_global_u4(void* p, vu4 v) {
#if defined(__HIP_DEVICE_COMPILE__)
  *reinterpret_cast<__attribute__((address_space(1))) vu4*>(reinterpret_cast<uintptr_t>(p)) = v;
#else
  *reinterpret_cast<vu4*>(p) = v;
#endif
}
__device__ __forceinline__ void store_global_u1(void* p, uint32_t v) {
#if defined(__HIP_DEVICE_COMPILE__)
  *reinterpret_cast<__attribute__((address_space(1))) uint32_t*>(reinterpret_cast<uintptr_t>(p)) = v;
#else
  *reinterpret_cast<uint32_t*>(p) = v;
#endif
}

struct K9Shared {
  float red_f[16];
  int64_t red_i[16];
  SelectShared sel;
};

// SQuant-E, SQuant-K and the candidate update for kernel Q (0..3) of a thread.
//   w       the thread's 36 weights; this kernel's are w[9Q .. 9Q+8]
//   packed  the thread's 36 output bytes as 9 dwords, biased codes (code + 128)
//   esum    += the kernel's Q24 perturbation sum after SQuant-K
//   cand_v  Q24 perturbation of the kernel's SQuant-C candidate (0 = none)
//   cand_b  its byte offset inside the thread's 36 output bytes
template <int Q, bool FAST_DIV>
__device__ __forceinline__ void k9_kernel_stage(const float (&w)[36], float s, float rs, float qmaxf, int mode,
                                                uint32_t (&packed)[9], int32_t& esum,
                                                int32_t& cand_v, int& cand_b) {
  float c[9];
  int32_t P[9];
#pragma unroll
  for (int i = 0; i < 9; ++i) {
    float x = FAST_DIV ? div_by_reciprocal(w[9 * Q + i], s, rs)
                       : w[9 * Q + i] / s;  // either way the IEEE binary32 quotient
    x = __builtin_amdgcn_fmed3f(x, -qmaxf, qmaxf);
    c[i] = rintf(x);
    const float p = c[i] - x;  // exact
    P[i] = __float2int_rn(p * 16777216.0f);
  }
  cand_v = 0;
  cand_b = 9 * Q;
  if (mode == SQUANT_MODE_E) {
#pragma unroll
    for (int i = 0; i < 9; ++i)
      packed[(9 * Q + i) >> 2] =
          __builtin_amdgcn_cvt_pk_u8_f32(c[i] + 128.0f, (9 * Q + i) & 3, packed[(9 * Q + i) >> 2]);
    return;
  }

  // ---- SQuant-K (Algorithm 2 on one kernel) ----
  int32_t E = 0;
#pragma unroll
  for (int i = 0; i < 9; ++i) E += P[i];
  const int32_t smask = E >> 31;                 // all ones when the sum is negative
  const int32_t A = (E ^ smask) - smask;         // |E|
  const int32_t k = (mode == SQUANT_MODE_EC) ? 0 : (int32_t)((uint32_t)(A + kHalf - 1) >> 24);
  const int32_t r = A - (k << 24);               // |sum| left after k flips, < 0: over SQuant
  esum += (r ^ smask) - smask;

  // unique keys: same-sign elements get (|p| - 1) << 4 | (15 - i) >= 0, all others < 0
  int32_t key[9], srt[9];
#pragma unroll
  for (int i = 0; i < 9; ++i) {
    const uint32_t a = (uint32_t)((P[i] ^ smask) + ~smask);
    key[i] = (int32_t)((a << 4) | (uint32_t)(15 - i));
    srt[i] = key[i];
  }
  top5_of_9(srt);
  int32_t s_km1 = 0x7fffffff, s_k = srt[0];      // (k-th, (k+1)-th) largest key, 1-based
  if (k >= 1) { s_km1 = srt[0]; s_k = srt[1]; }
  if (k >= 2) { s_km1 = srt[1]; s_k = srt[2]; }
  if (k >= 3) { s_km1 = srt[2]; s_k = srt[3]; }
  if (k >= 4) { s_km1 = srt[3]; s_k = srt[4]; }

  // flip the k largest: code -= sign(E); emit biased bytes
  const float keep = 128.0f;
  const float flip = smask ? 129.0f : 127.0f;
#pragma unroll
  for (int i = 0; i < 9; ++i) {
    const float cf = c[i] + (key[i] >= s_km1 ? flip : keep);
    packed[(9 * Q + i) >> 2] =
        __builtin_amdgcn_cvt_pk_u8_f32(cf, (9 * Q + i) & 3, packed[(9 * Q + i) >> 2]);
  }

  // ---- perturbation update (Algorithm 3): the kernel's candidate for SQuant-C ----
  const bool over = r < 0;
  const int32_t ck = over ? s_km1 : s_k;         // over: last flipped; under: first un-flipped
  if (ck >= 0) {
    const int32_t mag = (ck >> 4) + 1;           // |p| of that element before any flip
    const int32_t wv = mag - (over ? kOne : 0);  // over: post-flip value has the opposite sign
    cand_v = (wv ^ smask) - smask;
    cand_b = 9 * Q + 15 - (ck & 15);
  }
  if (E == 0) {
    // nothing is masked when the sum is exactly zero: largest |p| of either sign
    int32_t best = 0;
    cand_v = 0;
    cand_b = 9 * Q;
#pragma unroll
    for (int i = 0; i < 9; ++i) {
      const int32_t ap = P[i] < 0 ? -P[i] : P[i];
      if (ap > best) { best = ap; cand_v = P[i]; cand_b = 9 * Q + i; }
    }
  }
}

__global__ void __launch_bounds__(1024) squant_channel_k9(LaunchArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ K9Shared sh;

  int m;
  const TensorDesc d = locate(a, blockIdx.x, m);
  const int N = d.N, G = N >> 2;  // G threads carry kernels
  const int L = 9 * N, nvec = 9 * G;
  const int T = blockDim.x, tid = threadIdx.x;
  const float qmaxf = (float)a.qmax;
  vf4* stage = reinterpret_cast<vf4*>(smem);
  if (tid == 0) sh.sel.list_count = 0;

  // ---- stream the channel into LDS, 16 bytes per lane, fully coalesced ----
  // (the staging area holds 9*T vectors, so the stores need no bounds check; loads past the
  // end of the channel are clamped onto its last vector and land in the unused tail)
  {
    const float* src = d.w + (size_t)m * L;
    vf4 tmp[9];
#pragma unroll
    for (int j = 0; j < 9; ++j) {
      const int idx = tid + j * T;
      tmp[j] = load_global_f4(src + 4 * (idx < nvec ? idx : nvec - 1));
    }
#pragma unroll
    for (int j = 0; j < 9; ++j) stage[tid + j * T] = tmp[j];
  }
  __syncthreads();

  // ---- each thread takes its four kernels into registers ----
  float w[36];
  if (tid < G) {
#pragma unroll
    for (int j = 0; j < 9; ++j) {
      const vf4 q = stage[9 * tid + j];
      w[4 * j] = q.x; w[4 * j + 1] = q.y; w[4 * j + 2] = q.z; w[4 * j + 3] = q.w;
    }
  } else {
#pragma unroll
    for (int j = 0; j < 36; ++j) w[j] = 0.0f;
  }
  float amax = 0.0f;
#pragma unroll
  for (int j = 0; j < 36; j += 2) amax = fmaxf(fmaxf(amax, fabsf(w[j])), fabsf(w[j + 1]));
  amax = block_max_dpp(amax, sh.red_f);  // its barriers also retire every read of `stage`

  uint32_t* code32 = reinterpret_cast<uint32_t*>(smem);  // the staging area now holds codes
  int8_t* code8 = reinterpret_cast<int8_t*>(smem);
  const bool nonzero = amax > 0.0f;
  const float s = nonzero ? amax / qmaxf : 1.0f;
  if (tid == 0) d.scales[m] = s;

  int32_t esum = 0;
  int32_t cv[4] = {0, 0, 0, 0};
  int cb[4] = {0, 0, 0, 0};
  if (tid < G) {
    uint32_t packed[9];
#pragma unroll
    for (int j = 0; j < 9; ++j) packed[j] = 0;
    if (amax >= 0x1p-60f && amax <= 0x1p60f) {  // uniform over the workgroup
      const float rs = 1.0f / s;
      k9_kernel_stage<0, true>(w, s, rs, qmaxf, a.mode, packed, esum, cv[0], cb[0]);
      k9_kernel_stage<1, true>(w, s, rs, qmaxf, a.mode, packed, esum, cv[1], cb[1]);
      k9_kernel_stage<2, true>(w, s, rs, qmaxf, a.mode, packed, esum, cv[2], cb[2]);
      k9_kernel_stage<3, true>(w, s, rs, qmaxf, a.mode, packed, esum, cv[3], cb[3]);
    } else {
      k9_kernel_stage<0, false>(w, s, 0.0f, qmaxf, a.mode, packed, esum, cv[0], cb[0]);
      k9_kernel_stage<1, false>(w, s, 0.0f, qmaxf, a.mode, packed, esum, cv[1], cb[1]);
      k9_kernel_stage<2, false>(w, s, 0.0f, qmaxf, a.mode, packed, esum, cv[2], cb[2]);
      k9_kernel_stage<3, false>(w, s, 0.0f, qmaxf, a.mode, packed, esum, cv[3], cb[3]);
    }
#pragma unroll
    for (int j = 0; j < 9; ++j) code32[9 * tid + j] = packed[j] ^ 0x80808080u;
  }
  if (a.mode == SQUANT_MODE_EKC || a.mode == SQUANT_MODE_EC) {
    // ---- SQuant-C: every thread of the workgroup takes part ----
    const int64_t ec = block_sum_dpp(esum, sh.red_i);  // its barriers publish the codes
    const int sgn = sign_of(ec);
    const int64_t kc = flips_for(ec < 0 ? -ec : ec);
    if (kc > 0) {
      const int pos[4] = {36 * tid + cb[0], 36 * tid + cb[1], 36 * tid + cb[2], 36 * tid + cb[3]};
      channel_stage<4>(cv, pos, 4 * tid, sgn, (uint32_t)(kc > N ? N : kc), code8, sh.sel);
    }
  }
  __syncthreads();

  // ---- emit int8 codes, coalesced ----
  int8_t* out = d.codes + (size_t)m * L;
  if ((nvec & 3) == 0 && (reinterpret_cast<uintptr_t>(out) & 15u) == 0) {
    const vu4* src4 = reinterpret_cast<const vu4*>(smem);
    for (int j = tid; j < (nvec >> 2); j += T) store_global_u4(out + 16 * j, src4[j]);
  } else {
    for (int j = tid; j < nvec; j += T) store_global_u1(out + 4 * j, code32[j]);
  }
}

}  // namespace squant
