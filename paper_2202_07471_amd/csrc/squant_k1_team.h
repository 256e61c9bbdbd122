// SQuant kernel for short 1x1 / FC channels (cin <= 256, cin % 4 == 0): several output
// channels per wave.
//
// A channel of a few hundred bytes does not fill a wave, let alone a workgroup: with one
// wave per channel the fixed work of the wave (reductions, histogram scan, barriers)
// outweighs the channel's own, and a batch of such layers ran at 5-30 % of the memory
// bandwidth.  Here a TEAM of 4, 8 or 16 neighbouring lanes owns a channel, so a wave works
// on 16, 8 or 4 channels at once; a lane holds NV 16-byte vectors of its channel (lane l of
// the team has vectors l, l + TEAM, ...).  Every channel-wide step is a butterfly over the
// team's lanes with DPP (quad permutes, then the 8- and 16-lane mirrors): no LDS, no barrier,
// loads and stores fully coalesced, and all lanes of the wave run the same instructions.
//
// SQuant-C on such a channel (every element its own candidate, Section 3.4): the `need`
// largest |P| with the sign of the channel sum flip, lowest index first on ties.  With at
// most 256 candidates per team this is done by repeated arg-max: keys are
// (u << 8) | (255 - index) with u = |P| for the eligible elements (unique, so the maximum
// names one element and prefers the lower index among equal |P|); each step takes the
// team-wide maximum, the lane that holds it marks the element and clears the key.  The
// wave loops until every one of its teams has its `need` elements or runs out of
// candidates (typically 2-6 steps: need = round(|sum of cin perturbations|)).
#pragma once

#include "squant_common.h"
#include "squant_io.h"
#include "squant_plan.h"

namespace squant {

// Reductions over the TEAM (4, 8 or 16) lanes a lane belongs to; every lane gets the result.
template <int TEAM>
__device__ __forceinline__ float team_max_f32(float v) {
  v = fmaxf(v, dpp_f32<0xB1>(v));                   // quad_perm [1,0,3,2]
  v = fmaxf(v, dpp_f32<0x4E>(v));                   // quad_perm [2,3,0,1]
  if (TEAM >= 8) v = fmaxf(v, dpp_f32<0x141>(v));   // row_half_mirror
  if (TEAM >= 16) v = fmaxf(v, dpp_f32<0x140>(v));  // row_mirror
  return v;
}
template <int TEAM>
__device__ __forceinline__ uint32_t team_max_u32(uint32_t x) {
  int v = (int)x;
  v = (int)max((uint32_t)v, (uint32_t)dpp_i32<0xB1>(v));
  v = (int)max((uint32_t)v, (uint32_t)dpp_i32<0x4E>(v));
  if (TEAM >= 8) v = (int)max((uint32_t)v, (uint32_t)dpp_i32<0x141>(v));
  if (TEAM >= 16) v = (int)max((uint32_t)v, (uint32_t)dpp_i32<0x140>(v));
  return (uint32_t)v;
}
template <int TEAM>
__device__ __forceinline__ int32_t team_sum_i32(int32_t v) {  // |sum| < 2^31: cin <= 256, |P| <= 2^22
  v += dpp_i32<0xB1>(v);
  v += dpp_i32<0x4E>(v);
  if (TEAM >= 8) v += dpp_i32<0x141>(v);
  if (TEAM >= 16) v += dpp_i32<0x140>(v);
  return v;
}

// `item` is the workgroup's index within the tensor: it covers blockDim.x / TEAM channels.
template <int MODE, int TEAM, int NV>
__device__ __forceinline__ void k1_team_channels(const LaunchArgs& a, const TensorDesc& d, int item) {
  constexpr bool kChannelStage = MODE == SQUANT_MODE_EKC || MODE == SQUANT_MODE_EC;
  constexpr int NE = 4 * NV;
  const int tid = threadIdx.x;
  const int per_group = (int)blockDim.x / TEAM;
  const int l = tid & (TEAM - 1);  // lane within the team
  const int channel = item * per_group + tid / TEAM;
  const bool live = channel < d.M;
  const int c = live ? channel : d.M - 1;  // surplus teams shadow the last channel, store nothing
  const int N = d.N, nvec = N >> 2;
  const float qmaxf = (float)a.qmax;

  float w[NE];
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int idx = l + j * TEAM;
    const bool in = idx < nvec;
    const size_t at = (size_t)c * N + 4 * (size_t)(in ? idx : 0);
    float v0, v1, v2, v3;
    if (a.wtype == SQUANT_W_F32) {
      const vf4 v = load_global_f4(static_cast<const float*>(d.w) + at);
      v0 = v.x; v1 = v.y; v2 = v.z; v3 = v.w;
    } else {
      const uint32_t* p = reinterpret_cast<const uint32_t*>(static_cast<const uint16_t*>(d.w) + at);
      const bool bf16 = a.wtype == SQUANT_W_BF16;
      widen_pair(load_global_u1(p), bf16, v0, v1);
      widen_pair(load_global_u1(p + 1), bf16, v2, v3);
    }
    w[4 * j] = in ? v0 : 0.0f; w[4 * j + 1] = in ? v1 : 0.0f;
    w[4 * j + 2] = in ? v2 : 0.0f; w[4 * j + 3] = in ? v3 : 0.0f;
  }

  float amax = 0.0f;
#pragma unroll
  for (int e = 0; e < NE; ++e) amax = fmaxf(amax, fabsf(w[e]));
  amax = team_max_f32<TEAM>(amax);
  const float s = amax > 0.0f ? amax / qmaxf : 1.0f;
  if (live && l == 0) d.scales[channel] = s;
  // the reciprocal path only where every team of the wave is in its range (same quotients
  // either way; the choice must be the same for the whole wave)
  const bool fast = __ballot(!(amax >= 0x1p-60f && amax <= 0x1p60f) && amax > 0.0f) == 0ull;
  const float rs = 1.0f / s;

  float cf[NE];      // codes
  int32_t P[NE];     // perturbations, Q23
  int32_t esum = 0;
#pragma unroll
  for (int e = 0; e < NE; ++e) {
    const float x = fast ? div_by_reciprocal(w[e], s, rs) : w[e] / s;  // the IEEE quotient either way
    const float xc = __builtin_amdgcn_fmed3f(x, -qmaxf, qmaxf);
    cf[e] = rintf(xc);
    if (kChannelStage) {
      const float p = cf[e] - xc;  // exact
      P[e] = __float_as_int(__builtin_fmaf(p, 8388608.0f, 12582912.0f)) - 0x4B400000;
      esum += P[e];
    }
  }

  if (kChannelStage) {
    const int32_t ec = team_sum_i32<TEAM>(esum);
    const int32_t mag = ec < 0 ? -ec : ec;
    const int32_t kc = (int32_t)flips_for(mag);
    uint32_t need = (uint32_t)(kc > N ? N : kc);  // the same in every lane of a team
    const int32_t smask = ec >> 31;
    // unique keys: |P| above 255 - index for the elements with the sign of the sum, else 0
    uint32_t key[NE];
#pragma unroll
    for (int e = 0; e < NE; ++e) {
      const int32_t u = (P[e] ^ smask) - smask;  // P for a positive sum, -P for a negative one
      const int n = 4 * (l + (e >> 2) * TEAM) + (e & 3);
      key[e] = u > 0 ? ((uint32_t)u << 8) | (uint32_t)(255 - n) : 0u;
    }
    const float step = smask ? 1.0f : -1.0f;  // one step against the sum
    while (__ballot(need > 0) != 0ull) {
      uint32_t m = 0;
#pragma unroll
      for (int e = 0; e < NE; ++e) m = max(m, key[e]);
      m = team_max_u32<TEAM>(m);
      const bool take = need > 0 && m != 0;
#pragma unroll
      for (int e = 0; e < NE; ++e) {
        const bool hit = take && key[e] == m;
        cf[e] += hit ? step : 0.0f;
        key[e] = hit ? 0u : key[e];
      }
      need = take ? need - 1 : 0u;  // out of candidates: this team is done
    }
  }

  if (!live) return;
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int idx = l + j * TEAM;
    if (idx >= nvec) continue;
    const size_t at = (size_t)channel * N + 4 * (size_t)idx;  // first element of this vector
    if (a.out_format == SQUANT_OUT_INT8) {
      uint32_t packed = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) packed = __builtin_amdgcn_cvt_pk_u8_f32(cf[4 * j + e] + 128.0f, e, packed);
      store_global_u1(static_cast<int8_t*>(d.out) + at, packed ^ 0x80808080u);
    } else if (a.out_format == SQUANT_OUT_INT4) {
      uint32_t packed = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) packed |= ((uint32_t)(int)cf[4 * j + e] & 0xFu) << (4 * e);
      store_global_u16(static_cast<uint8_t*>(d.out) + (size_t)channel * (N / 2) + 2 * (size_t)idx,
                       (uint16_t)packed);
    } else if (a.out_format == SQUANT_OUT_BF16) {
      uint16_t* out = static_cast<uint16_t*>(d.out) + at;
#pragma unroll
      for (int e = 0; e < 4; ++e) out[e] = (uint16_t)bf16_bits((cf[4 * j + e] + 0.0f) * s);  // code -0 is 0
    } else {  // SQUANT_OUT_F32
      float* out = static_cast<float*>(d.out) + at;
#pragma unroll
      for (int e = 0; e < 4; ++e) out[e] = (cf[4 * j + e] + 0.0f) * s;  // code -0 is 0
    }
  }
}

// Picks TEAM and NV from cin (<= kMaxTeamCin): the smallest team whose lanes hold the channel
// with one vector each, then 16 lanes with two or four vectors.
template <int MODE>
__device__ __forceinline__ void k1_team_dispatch(const LaunchArgs& a, const TensorDesc& d, int item) {
  const int N = d.N;
  if (N <= 16) k1_team_channels<MODE, 4, 1>(a, d, item);
  else if (N <= 32) k1_team_channels<MODE, 8, 1>(a, d, item);
  else if (N <= 64) k1_team_channels<MODE, 16, 1>(a, d, item);
  else if (N <= 128) k1_team_channels<MODE, 16, 2>(a, d, item);
  else k1_team_channels<MODE, 16, 4>(a, d, item);
}

// Compiled for eight waves per SIMD (64 VGPRs instead of 66: measured 1-4 % faster).
template <int MODE>
__global__ void __launch_bounds__(256)
    __attribute__((amdgpu_waves_per_eu(8))) squant_channel_k1_team(LaunchArgs a) {
  int m;
  const TensorDesc d = locate(a, blockIdx.x, m);
  k1_team_dispatch<MODE>(a, d, m);
}

}  // namespace squant
