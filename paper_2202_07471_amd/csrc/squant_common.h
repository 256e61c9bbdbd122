// Shared device-side definitions of the SQuant gfx950 kernels: tensor descriptors,
// SQuant-E arithmetic, wave / workgroup reductions.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "squant.h"
#include "squant_arith.h"

namespace squant {


constexpr int32_t kOne = 1 << 23;   // 1.0 in Q23
constexpr int32_t kHalf = 1 << 22;  // 0.5 in Q23
constexpr int kWave = 64;
constexpr int kXcdRun = 64;  // consecutive channels one XCD takes at a time (see locate)

struct TensorDesc {
  const void* w;  // weights, in the launch's weight type
  void* out;      // codes or dequantised weights, in the launch's output format
  float* scales;
  int32_t M, N, K;
  int32_t first;  // this tensor's first workgroup within its launch
};

// The tensor descriptors of a launch travel inside the kernel arguments (10 KB for 256 of
// them, read with scalar loads); a batch of more tensors takes several launches.
constexpr int kInlineDescs = 256;

struct LaunchArgs {
  int32_t n_tensors;        // descriptors in `table`, ordered by `first`
  int32_t total;            // workgroups in this launch (one per output channel, except depthwise)
  int32_t uniform_m;        // > 0: every tensor of the table takes this many workgroups
  int32_t uniform_shift;    // >= 0: uniform_m == 1 << uniform_shift
  int32_t qmax;
  int32_t mode;
  int32_t out_format;       // squant_output_t
  int32_t wtype;            // squant_wtype_t
  int32_t wave_span;        // channels a wave of the wave-per-channel 1x1 routine walks
  TensorDesc table[kInlineDescs];
};

// ---------------------------------------------------------------------------
// small device helpers
// ---------------------------------------------------------------------------

__device__ __forceinline__ TensorDesc locate(const LaunchArgs& a, int g, int& m) {
  // Workgroups are dealt to the 8 XCDs round robin.  Re-deal them so that every XCD works on
  // runs of kXcdRun consecutive channels (consecutive memory): within each group of
  // 8 * kXcdRun workgroups, XCD x takes channels x * kXcdRun .. x * kXcdRun + kXcdRun - 1.
  // The tail that does not fill a group keeps its order.  Measured 1 % faster on the large
  // 3x3 workload with runs of 64 to 256, neutral elsewhere; whole eighths gain nothing.
  {
    constexpr int group = 8 * kXcdRun;
    if (g < a.total - a.total % group) {
      const int r = g % group;
      g = g - r + (r & 7) * kXcdRun + (r >> 3);
    }
  }
  int t = 0;
  if (a.n_tensors > 1) {
    if (a.uniform_shift >= 0) {
      t = g >> a.uniform_shift;
    } else if (a.uniform_m > 0) {
      t = g / a.uniform_m;
    } else {
      // last t with first[t] <= g.  The offsets ascend, so t + 1 is the number of tensors whose
      // first workgroup is <= g: every lane fetches one offset (64 per step, one memory latency
      // instead of the chain of dependent loads of a binary search) and a ballot counts them.
      const int lane = threadIdx.x & (kWave - 1);
      int below = 0;
      for (int base = 0; base < a.n_tensors; base += kWave) {
        const int i = base + lane;
        const int first = i < a.n_tensors ? a.table[i].first : 0x7fffffff;
        const int cnt = __popcll(__ballot(first <= g));
        below += cnt;
        if (cnt < kWave) break;
      }
      t = __builtin_amdgcn_readfirstlane(below - 1);
    }
  }
  const TensorDesc d = a.table[t];
  m = g - d.first;
  return d;
}

__device__ __forceinline__ int sign_of(int64_t v) { return (v > 0) - (v < 0); }

// k = round(|e|), an exact half rounded down (Algorithm 2, "k = round(|e|)").
__device__ __forceinline__ int64_t flips_for(int64_t abs_sum) { return (abs_sum + kHalf - 1) >> 23; }

// SQuant-E on one scaled weight (Algorithm 1, rounding and element perturbation):
// returns the integer code, writes the Q23 perturbation code - x.
__device__ __forceinline__ int round_and_perturb(float w, float s, float qmaxf, int32_t& P) {
  float x = w / s;  // IEEE binary32 division
  x = fminf(fmaxf(x, -qmaxf), qmaxf);
  const float c = rintf(x);  // round half to even
  const float p = c - x;     // exact
  P = __float2int_rn(p * 8388608.0f);
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

// ---- DPP reductions (wave64 = 4 rows of 16 lanes) ----
// After the four steps every lane of a row holds the row's result; the four row
// results are then read as scalars.  DPP controls: quad_perm [1,0,3,2] = 0xB1,
// quad_perm [2,3,0,1] = 0x4E, row_half_mirror = 0x141, row_mirror = 0x140.
template <int CTRL>
__device__ __forceinline__ int dpp_i32(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, false);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}

// max over the wave of non-negative floats; uniform result.  The bit patterns of non-negative
// floats order like unsigned integers, and the integer maximum folds into the DPP move.
__device__ __forceinline__ float wave_max_dpp(float v) {
  uint32_t u = __float_as_uint(v);
  u = max(u, (uint32_t)dpp_i32<0xB1>((int)u));
  u = max(u, (uint32_t)dpp_i32<0x4E>((int)u));
  u = max(u, (uint32_t)dpp_i32<0x141>((int)u));
  u = max(u, (uint32_t)dpp_i32<0x140>((int)u));
  const uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)u, 0);
  const uint32_t r1 = (uint32_t)__builtin_amdgcn_readlane((int)u, 16);
  const uint32_t r2 = (uint32_t)__builtin_amdgcn_readlane((int)u, 32);
  const uint32_t r3 = (uint32_t)__builtin_amdgcn_readlane((int)u, 48);
  return __uint_as_float(max(max(r0, r1), max(r2, r3)));
}

// sum over the wave of any int32 values; uniform 64-bit result.  The low 16 bits (unsigned) and
// the high 16 bits (signed) are added up separately, so no partial sum leaves 32 bits.
__device__ __forceinline__ int32_t wave_sum_dpp_small(int32_t v) {  // |v| <= 2^24
  v += dpp_i32<0xB1>(v);
  v += dpp_i32<0x4E>(v);
  v += dpp_i32<0x141>(v);
  v += dpp_i32<0x140>(v);
  return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) +
         __builtin_amdgcn_readlane(v, 32) + __builtin_amdgcn_readlane(v, 48);
}
__device__ __forceinline__ int64_t wave_sum_dpp(int32_t v) {
  const int32_t lo = wave_sum_dpp_small(v & 0xFFFF);
  const int32_t hi = wave_sum_dpp_small(v >> 16);
  return (int64_t)hi * 65536 + lo;
}

// Running maximum over the lanes of a wave: lane 63 ends up with the wave's maximum (same
// DPP steps as a prefix sum).
__device__ __forceinline__ uint32_t wave_prefix_max_u32(uint32_t x) {
  int v = (int)x;
  v = (int)max((uint32_t)v, (uint32_t)__builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true));
  v = (int)max((uint32_t)v, (uint32_t)__builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true));
  v = (int)max((uint32_t)v, (uint32_t)__builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true));
  v = (int)max((uint32_t)v, (uint32_t)__builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true));
  v = (int)max((uint32_t)v, (uint32_t)__builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false));
  v = (int)max((uint32_t)v, (uint32_t)__builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false));
  return (uint32_t)v;
}

// Workgroup-wide versions: every thread returns the result.  `slot` holds >= 16 entries.
// One barrier each: for callers that pass at least one other workgroup barrier before they
// reduce into the same slots again (so no wave can still be reading them).
__device__ __forceinline__ float block_max_dpp1(float v, float* slot) {
  v = wave_max_dpp(v);
  const int wid = threadIdx.x / kWave, nw = (blockDim.x + kWave - 1) / kWave;
  if ((threadIdx.x & (kWave - 1)) == 0) slot[wid] = v;
  __syncthreads();
  float r = slot[0];
  for (int i = 1; i < nw; ++i) r = fmaxf(r, slot[i]);
  return r;
}

__device__ __forceinline__ int64_t block_sum_dpp1(int32_t v, int64_t* slot) {
  const int64_t w = wave_sum_dpp(v);
  const int wid = threadIdx.x / kWave, nw = (blockDim.x + kWave - 1) / kWave;
  if ((threadIdx.x & (kWave - 1)) == 0) slot[wid] = w;
  __syncthreads();
  int64_t r = slot[0];
  for (int i = 1; i < nw; ++i) r += slot[i];
  return r;
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
