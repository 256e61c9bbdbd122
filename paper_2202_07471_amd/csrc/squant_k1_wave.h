// SQuant kernel for 1x1 convolutions and fully connected layers whose channel fits one wave
// (256 < cin <= 2048, cin % 4 == 0): one wave per output channel, several channels per wave.
//
// A channel of one or two thousand weights keeps a wave busy for about a microsecond, most of
// it waiting: for its weights, then for the steps of the channel stage, which follow each
// other.  A workgroup per channel pays that wait once per channel and a workgroup launch on
// top.  Here a wave walks `span` consecutive channels (four in a launch large enough to keep
// the chip full that way, else one) and, PREFETCH, asks for the next channel's weights as soon
// as SQuant-E has consumed the current ones, so the loads travel while the wave selects the
// current channel's flips; the waves of a workgroup work on neighbouring runs of channels and
// never meet (no workgroup barrier, every wave has its own selection area in LDS).
//
// The arithmetic and the selection are those of the workgroup kernel (squant_k1.h) with the
// wave's lanes as the threads: lane l holds vectors l, l + 64, ... of the channel.
#pragma once

#include "squant_k1.h"
#include "squant_plan.h"

namespace squant {

// A wave's selection area: the members of SelectShared that the one-element selection uses,
// with the histogram cut to its 260 bins, and the lanes' owner masks.
struct alignas(16) K1WaveSel {
  uint32_t hist[264];  // 257 bins and the scan's padding; 264 = 66 x 16 bytes
  uint32_t list_count;
  uint32_t pad_[3];  // keeps the lists on 16 bytes
  uint32_t list_key[kListCap];
  uint32_t list_n[kListCap];
  uint32_t wave_cnt[20];
  uint32_t owner[kWave];
};

template <int MODE, int NV, bool PREFETCH>
__device__ __forceinline__ void k1_wave_channels(const LaunchArgs& a, const TensorDesc& d, int c0, int c1,
                                                 K1WaveSel& sel) {
  constexpr bool kChannelStage = MODE == SQUANT_MODE_EKC || MODE == SQUANT_MODE_EC;
  constexpr int NE = 4 * NV;
  const float qmaxf = (float)a.qmax;
  const int N = d.N, nvec = N >> 2;  // cin % 4 == 0

  float w[NE];
  auto load_channel = [&](int m, int lane) {
    if (a.wtype == SQUANT_W_F32) {
      const float* src = static_cast<const float*>(d.w) + (size_t)m * N;
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        const int idx = lane + j * kWave;
        vf4 v = {0.0f, 0.0f, 0.0f, 0.0f};
        if (idx < nvec) v = load_global_f4_stream(src + 4 * idx);
        w[4 * j] = v.x; w[4 * j + 1] = v.y; w[4 * j + 2] = v.z; w[4 * j + 3] = v.w;
      }
    } else {  // 16-bit weights: the same four elements per vector, 8 bytes
      const uint16_t* src = static_cast<const uint16_t*>(d.w) + (size_t)m * N;
      const bool bf16 = a.wtype == SQUANT_W_BF16;
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        const int idx = lane + j * kWave;
        vu2 v = {0u, 0u};
        if (idx < nvec) v = load_global_u2_stream(src + 4 * idx);
        widen_pair(v.x, bf16, w[4 * j], w[4 * j + 1]);
        widen_pair(v.y, bf16, w[4 * j + 2], w[4 * j + 3]);
      }
    }
  };

  if (PREFETCH && c0 < c1) load_channel(c0, k1_tid<true>());
#pragma unroll 1
  for (int m = c0; m < c1; ++m) {
    const int lane = k1_tid<true>();  // taken anew in every round, see k1_tid
    if (!PREFETCH) load_channel(m, lane);
    if (kChannelStage) {  // the area is free: the previous channel's last LDS access precedes these
      for (int b = lane; b < 66; b += kWave) reinterpret_cast<uint4*>(sel.hist)[b] = make_uint4(0, 0, 0, 0);
      if (lane == 0) sel.list_count = 0;
      k1_list_reset<true>(sel);
      sel.owner[lane] = 0;
    }
    float amax = 0.0f;
#pragma unroll
    for (int e = 0; e < NE; e += 2) amax = fmaxf(fmaxf(amax, fabsf(w[e])), fabsf(w[e + 1]));
    amax = wave_max_dpp(amax);
    const float s = amax > 0.0f ? amax / qmaxf : 1.0f;
    if (lane == 0) d.scales[m] = s;

    // ---- SQuant-E (Algorithm 1): codes and perturbations in registers ----
    int32_t esum = 0;
    uint32_t B[NE];
    uint32_t code[NV];
    {
      const bool prescale = !(amax <= 0x1p60f && (amax >= 0x1p-60f || amax == 0.0f));
      const float f1 = !prescale ? 1.0f : amax < 1.0f ? 0x1p64f : 0x1p-64f;
      const float a1 = amax * f1;
      const float f2 = !prescale ? 1.0f : a1 < 0x1p-60f ? 0x1p64f : a1 > 0x1p60f ? 0x1p-64f : 1.0f;
      const float s2 = s * f1 * f2;
      k1_round_all<NV, kChannelStage>(w, s2, 1.0f / s2, qmaxf, prescale, f1, f2, code, B, esum);
    }
    // the weights are used up: the next channel's travel while this one's flips are chosen
    if (PREFETCH && m + 1 < c1) load_channel(m + 1, lane);

    if (kChannelStage) {
      k1_sync<true>();  // the area is reset
#pragma unroll
      for (int j = 0; j < NV; ++j)
        if (lane + j * kWave < nvec) {  // idle elements stay out of the histogram (see squant_k1.h)
#pragma unroll
          for (int e = 0; e < 4; ++e) k1_count_biased(sel, B[4 * j + e]);
        }
      const int64_t ec = wave_sum_dpp(esum);
      k1_sync<true>();  // the histogram is complete
      const int sgn = sign_of(ec);
      const int64_t kc = flips_for(ec < 0 ? -ec : ec);
      if (kc > 0) {
        const uint32_t flip =
            k1_channel_stage<NE, uint32_t, true>(B, sgn, (uint32_t)(kc > N ? N : kc), sel, sel.owner);
        const uint32_t sm = sgn < 0 ? ~0u : 0u;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
          const uint32_t f4 = (flip >> (4 * j)) & 15u;
          const uint32_t b = (f4 * 0x204081u) & 0x01010101u;  // bit e to byte e
          code[j] -= (b ^ sm) - sm;
        }
      }
      k1_sync<true>();  // the channel's last LDS access
    }

    auto emit_all = [&](int format) {
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        const int idx = lane + j * kWave;
        if (idx < nvec) k1_emit_vector(code[j], idx, d.out, m, N, s, format);
      }
    };
    if (a.out_format == SQUANT_OUT_INT8) emit_all(SQUANT_OUT_INT8);
    else if (a.out_format == SQUANT_OUT_INT4) emit_all(SQUANT_OUT_INT4);
    else if (a.out_format == SQUANT_OUT_BF16) emit_all(SQUANT_OUT_BF16);
    else emit_all(SQUANT_OUT_F32);
  }
}

// `item` is the workgroup's index within the tensor: each of its waves takes a.wave_span
// channels.  smem: one K1WaveSel per wave.
template <int MODE, int NV, bool PREFETCH>
__device__ __forceinline__ void k1_wave_item(const LaunchArgs& a, const TensorDesc& d, int item,
                                             unsigned char* smem) {
  const int wave = threadIdx.x / kWave, waves = blockDim.x / kWave;
  const int c0 = (item * waves + wave) * a.wave_span;
  const int c1 = c0 + a.wave_span < d.M ? c0 + a.wave_span : d.M;
  k1_wave_channels<MODE, NV, PREFETCH>(a, d, c0, c1, reinterpret_cast<K1WaveSel*>(smem)[wave]);
}

// For the mixed kernel: vectors per lane from the channel's length, 2 to 8; without the
// prefetch, whose registers that kernel does not have.
template <int MODE>
__device__ __forceinline__ void k1_wave_dispatch(const LaunchArgs& a, const TensorDesc& d, int item,
                                                 unsigned char* smem) {
  switch ((d.N / 4 + kWave - 1) / kWave) {
    case 2: k1_wave_item<MODE, 2, false>(a, d, item, smem); break;
    case 3: k1_wave_item<MODE, 3, false>(a, d, item, smem); break;
    case 4: k1_wave_item<MODE, 4, false>(a, d, item, smem); break;
    case 5: k1_wave_item<MODE, 5, false>(a, d, item, smem); break;
    case 6: k1_wave_item<MODE, 6, false>(a, d, item, smem); break;
    case 7: k1_wave_item<MODE, 7, false>(a, d, item, smem); break;
    default: k1_wave_item<MODE, 8, false>(a, d, item, smem); break;
  }
}

// One kernel per vector count.  The next channel's weights share the registers with the
// current channel's perturbations and codes, about 9 per vector and 25 besides: two vectors fit
// the 64 VGPRs of eight waves per SIMD, four the 80 of six, six the 96 of five, eight the 128 of
// four.  (Four vectors in 80 registers and six in 96 spill 12 and 32 bytes; the next step down
// in waves was measured 2 to 4 points of the roofline slower.)
template <int MODE, int NV>
__global__ void __launch_bounds__(256)
    __attribute__((amdgpu_waves_per_eu(NV <= 2 ? 8 : NV <= 4 ? 6 : NV <= 6 ? 5 : 4)))
    squant_channel_k1_wave(LaunchArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];  // one K1WaveSel per wave
  int item;
  const TensorDesc d = locate(a, blockIdx.x, item);
  k1_wave_item<MODE, NV, true>(a, d, item, smem);
}

}  // namespace squant
