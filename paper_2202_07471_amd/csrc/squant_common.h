// Shared device-side definitions of the SQuant gfx950 kernels: tensor descriptors,
// SQuant-E arithmetic, wave / workgroup reductions.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "squant.h"

namespace squant {


constexpr int32_t kOne = 1 << 24;   // 1.0 in Q24
constexpr int32_t kHalf = 1 << 23;  // 0.5 in Q24
constexpr int kWave = 64;

struct TensorDesc {
  const float* w;
  int8_t* codes;
  float* scales;
  int32_t M, N, K;
  int32_t first;  // index of this tensor's channel 0 within its launch
};

struct LaunchArgs {
  TensorDesc single;        // used when table == nullptr
  const TensorDesc* table;  // device table, n_tensors entries ordered by `first`
  int32_t n_tensors;
  int32_t uniform_m;        // > 0: every tensor of the table has this many channels
  int32_t qmax;
  int32_t mode;
};

// ---------------------------------------------------------------------------
// small device helpers
// ---------------------------------------------------------------------------

__device__ __forceinline__ TensorDesc locate(const LaunchArgs& a, int g, int& m) {
  if (a.table == nullptr) {
    m = g;
    return a.single;
  }
  int t;
  if (a.uniform_m > 0) {
    t = g / a.uniform_m;
  } else {  // last t with first[t] <= g
    int lo = 0, hi = a.n_tensors - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (a.table[mid].first <= g) lo = mid; else hi = mid - 1;
    }
    t = lo;
  }
  const TensorDesc d = a.table[t];
  m = g - d.first;
  return d;
}

__device__ __forceinline__ int sign_of(int64_t v) { return (v > 0) - (v < 0); }

// k = round(|e|), an exact half rounded down (Algorithm 2, "k = round(|e|)").
__device__ __forceinline__ int64_t flips_for(int64_t abs_sum) { return (abs_sum + kHalf - 1) >> 24; }

// SQuant-E on one scaled weight (Algorithm 1, rounding and element perturbation):
// returns the integer code, writes the Q24 perturbation code - x.
__device__ __forceinline__ int round_and_perturb(float w, float s, float qmaxf, int32_t& P) {
  float x = w / s;  // IEEE binary32 division
  x = fminf(fmaxf(x, -qmaxf), qmaxf);
  const float c = rintf(x);  // round half to even
  const float p = c - x;     // exact
  P = __float2int_rn(p * 16777216.0f);
  return (int)c;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  return v;
}

__device__ __forceinline__ int64_t wave_sum(int64_t v) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

// Every thread returns the block-wide result.  `slot` holds >= 16 entries.
__device__ __forceinline__ float block_max(float v, float* slot) {
  v = wave_max(v);
  const int wid = threadIdx.x / kWave, nw = (blockDim.x + kWave - 1) / kWave;
  __syncthreads();
  if ((threadIdx.x & (kWave - 1)) == 0) slot[wid] = v;
  __syncthreads();
  float r = slot[0];
  for (int i = 1; i < nw; ++i) r = fmaxf(r, slot[i]);
  return r;
}

__device__ __forceinline__ int64_t block_sum(int64_t v, int64_t* slot) {
  v = wave_sum(v);
  const int wid = threadIdx.x / kWave, nw = (blockDim.x + kWave - 1) / kWave;
  __syncthreads();
  if ((threadIdx.x & (kWave - 1)) == 0) slot[wid] = v;
  __syncthreads();
  int64_t r = slot[0];
  for (int i = 1; i < nw; ++i) r += slot[i];
  return r;
}

}  // namespace squant
