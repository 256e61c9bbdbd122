// One launch for a set of layers of different shapes (the weight tensors of a network are
// independent problems, Section 4.2).  Every workgroup finds its tensor and output channel
// in the descriptor table, picks the tensor's kernel variant the same way the host did and
// runs that variant's channel routine.  The workgroup size is the largest any member tensor
// needs (at most 256); the routines let surplus threads idle.
#pragma once

#include "squant_generic.h"
#include "squant_k1.h"
#include "squant_k1_team.h"
#include "squant_k1_wave.h"
#include "squant_k9.h"
#include "squant_plan.h"

namespace squant {

constexpr int kMixedMaxThreads = 256;

// Compiled for five waves per SIMD (at most 96 VGPRs, what the four-kernel 3x3 routine needs):
// these launches live on the number of resident workgroups.  Measured 2-4 % faster on the
// ResNet-50 and MobileNetV2 sets; eight waves spill in the 3x3 routine and cost ResNet-18 24 %.
template <int MODE>
__global__ void __launch_bounds__(kMixedMaxThreads)
    __attribute__((amdgpu_waves_per_eu(5))) squant_channel_mixed(LaunchArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ K9Shared sh;
  __shared__ GenericShared gs;
  // one-element kernels: E&K is E and E&C is E&K&C (SQuant-K has nothing to do, Section 3.4)
  constexpr int M1 = (MODE == SQUANT_MODE_EK) ? SQUANT_MODE_E
                     : (MODE == SQUANT_MODE_EC) ? SQUANT_MODE_EKC : MODE;
  int m;
  const TensorDesc d = locate(a, blockIdx.x, m);
  // Per-thread work is chosen from the launch's workgroup size T, not from the variant the
  // tensor would get in a launch of its own: as few kernels / vectors per thread as T allows.
  // The host only admits tensors with cin <= 4T (3x3) or cin <= 16T (1x1).
  const int T = blockDim.x;
  const int family = choose_family(d.N, d.K, pointers_aligned(d.w, d.out));
  if (family == 9) {
    if (d.N <= T) k9_channel<MODE, 1>(a, d, m, smem, sh);
    else if (d.N <= 2 * T) k9_channel<MODE, 2>(a, d, m, smem, sh);
    else k9_channel<MODE, 4>(a, d, m, smem, sh);
  } else if (family == 1) {
    const int nvec = d.N >> 2;
    if (nvec <= T) k1_channel<M1, 1>(a, d, m, smem, sh);
    else if (nvec <= 2 * T) k1_channel<M1, 2>(a, d, m, smem, sh);
    else if (nvec <= 3 * T) k1_channel<M1, 3>(a, d, m, smem, sh);
    else k1_channel<M1, 4>(a, d, m, smem, sh);
  } else if (family == 3) {
    dw9_channels<MODE>(a, d, m);
  } else if (family == 4) {
    k1_team_dispatch<M1>(a, d, m);
  } else if (family == 6) {
    k1_wave_dispatch<M1>(a, d, m, smem);
  } else {
    generic_channel(a, d, m, smem, gs);
  }
}

}  // namespace squant
