// Activation ranges from batch-norm parameters (Section 4, experimental set-up): one
// workgroup per layer reduces beta_c -/+ n_sigma * |gamma_c| over the layer's channels and
// derives the uniform quantizer of the resulting per-tensor range.
#pragma once

#include "squant_common.h"

namespace squant {

struct BnDesc {
  const float* gamma;
  const float* beta;
  int32_t channels;
  int32_t relu;
  int32_t out_index;  // entry of the result array this layer writes
  int32_t pad_;
};

// The layer descriptors of a launch travel in the kernel arguments (8 KB for 256 layers).
constexpr int kInlineBn = 256;
struct BnArgs {
  float n_sigma;
  int32_t levels_minus_1;
  squant_act_range_t* out;
  BnDesc layer[kInlineBn];
};

__global__ void __launch_bounds__(256) squant_activation_range_kernel(BnArgs a) {
  __shared__ float red_lo[16], red_hi[16];
  const BnDesc d = a.layer[blockIdx.x];
  const float n_sigma = a.n_sigma;
  const int32_t levels_minus_1 = a.levels_minus_1;
  squant_act_range_t* out = a.out;
  float lo = INFINITY, hi = -INFINITY;
  for (int c = threadIdx.x; c < d.channels; c += blockDim.x) {
    const float t = n_sigma * fabsf(d.gamma[c]);
    const float b = d.beta[c];
    lo = fminf(lo, b - t);
    hi = fmaxf(hi, b + t);
  }
  lo = -block_max(-lo, red_lo);
  hi = block_max(hi, red_hi);
  if (threadIdx.x == 0) {
    if (d.relu) { lo = fmaxf(lo, 0.0f); hi = fmaxf(hi, 0.0f); }
    lo += 0.0f;  // a zero bound is +0
    hi += 0.0f;
    squant_act_range_t r;
    r.lo = lo;
    r.hi = hi;
    const float span = hi - lo;
    const float q = (float)levels_minus_1;
    r.scale = span > 0.0f ? span / q : 1.0f;
    float z = rintf(-lo / r.scale);
    z = fminf(fmaxf(z, 0.0f), q);
    r.zero_point = (int32_t)z;
    out[d.out_index] = r;
  }
}

}  // namespace squant
