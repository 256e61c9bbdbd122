// SQuant kernel for 1x1 convolutions and fully connected layers (K = kh*kw = 1).
//
// With one element per kernel SQuant-K has nothing to do (k = round(|p|) = 0 for |p| <= 0.5,
// Section 3.4), every element is its own kernel, and its rounding perturbation is its
// SQuant-C candidate (Algorithm 3, "under SQuant" with k = 0).  One workgroup per output
// channel; a thread takes NV 16-byte vectors of the channel, vector j of thread t being
// vector t + j*T, so every load instruction of a wave reads 1 KB of consecutive weights.
// SQuant-E runs in registers, the int8 codes go to LDS four to a dword, and SQuant-C is an
// LDS radix select over the signed perturbations of all cin elements of the channel.
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

// ---------------------------------------------------------------------------
// SQuant-C for one-element kernels.  Every element is a candidate and its candidate value is
// its own rounding perturbation P (Q23, |P| <= 2^22), so the selection works on P directly:
// the `need` elements with the largest |P| among those with the sign of the channel sum,
// lowest index first on ties.  A radix select over the signed value:
//   level 0  257 bins of P >> 15, counted into LDS before the channel sum (and with it the
//            wanted sign) is known: negative P in bins 0..127, P >= 0 in bins 128..256.  The
//            scan runs from the outside in over the wanted sign's bins only.
//   below    u = P (sum > 0) or ~P (sum < 0) orders the wanted side "larger is better";
//            bits 14..7 and 7..0 of u get a 256-bin pass each while the boundary bin still
//            holds more keys than the ranking list takes.
// A thread keeps the elements still undecided as a bit mask.  P = 0 is no candidate but
// shares bin 128 with small positive P: when the scan ends in that bin the members are
// counted again exactly.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void k1_count(SelectShared& sh, int32_t P) {
  atomicAdd(&sh.hist[(P >> 15) + 128], 1u);
}

// Level 0 scan, by every wave on its own.  Returns the boundary bin in u units
// (d = u >> 15 of the need-th best key, 0..128), or -1 when the wanted side holds fewer than
// `need` keys; need_at = keys still wanted inside that bin, count_at = keys in it.
__device__ __forceinline__ int k1_scan_top(const uint32_t* hist, int sgn, uint32_t need,
                                           uint32_t& need_at, uint32_t& count_at) {
  const int lane = threadIdx.x & (kWave - 1);
  // traversal order: sum > 0 from bin 259 (padding) down to 128, sum < 0 from bin 0 up to 127
  const bool on = sgn > 0 ? lane <= 32 : lane <= 31;
  const int quad = sgn > 0 ? 64 - lane : lane;
  uint4 h = make_uint4(0, 0, 0, 0);
  if (on) h = reinterpret_cast<const uint4*>(hist)[quad];
  const uint32_t a0 = sgn > 0 ? h.w : h.x, a1 = sgn > 0 ? h.z : h.y;
  const uint32_t a2 = sgn > 0 ? h.y : h.z, a3 = sgn > 0 ? h.x : h.w;
  const uint32_t mine = a0 + a1 + a2 + a3;
  const uint32_t incl = wave_prefix_sum(mine);
  const unsigned long long reach = __ballot(incl >= need);
  if (reach == 0ull) { need_at = 0; count_at = 0; return -1; }
  const int l = __builtin_ctzll(reach);
  const uint32_t above = (uint32_t)__builtin_amdgcn_readlane((int)(incl - mine), l);
  const uint32_t b0 = (uint32_t)__builtin_amdgcn_readlane((int)a0, l);
  const uint32_t b1 = (uint32_t)__builtin_amdgcn_readlane((int)a1, l);
  const uint32_t b2 = (uint32_t)__builtin_amdgcn_readlane((int)a2, l);
  const uint32_t b3 = (uint32_t)__builtin_amdgcn_readlane((int)a3, l);
  int t = 4 * l;  // position in traversal order
  if (above + b0 >= need) { need_at = need - above; count_at = b0; }
  else if (above + b0 + b1 >= need) { need_at = need - above - b0; count_at = b1; t += 1; }
  else if (above + b0 + b1 + b2 >= need) { need_at = need - above - b0 - b1; count_at = b2; t += 2; }
  else { need_at = need - above - b0 - b1 - b2; count_at = b3; t += 3; }
  // bin index = 259 - t (sum > 0) or t (sum < 0); u >> 15 = bin - 128 resp. ~(bin - 128)
  return (sgn > 0 ? 131 : 127) - t;
}

// Ranks the `count` (key, index) pairs of the list against each other: larger key first, then
// lower index; the first `need` flip.  Four lanes share a pair, each comparing it with every
// fourth group of four list entries (two 16-byte LDS reads per group), and add their counts
// up inside the quad.  Slots past `count` hold (0, 0xFFFFFFFF), which ranks below every pair.
// After a barrier that follows the last push.
__device__ __forceinline__ void k1_rank_list(SelectShared& sh, uint32_t count, uint32_t need, int sgn,
                                             uint32_t* code32) {
  const uint32_t sub = threadIdx.x & 3u, groups = (count + 3u) >> 2;
  const uint4* key4 = reinterpret_cast<const uint4*>(sh.list_key);
  const uint4* n4 = reinterpret_cast<const uint4*>(sh.list_n);
  for (uint32_t i = threadIdx.x >> 2; i < count; i += blockDim.x >> 2) {
    const uint32_t key = sh.list_key[i], n = sh.list_n[i];
    int rank = 0;
    for (uint32_t g = sub; g < groups; g += 4) {
      const uint4 ek = key4[g], en = n4[g];
      rank += (ek.x > key || (ek.x == key && en.x < n)) ? 1 : 0;
      rank += (ek.y > key || (ek.y == key && en.y < n)) ? 1 : 0;
      rank += (ek.z > key || (ek.z == key && en.z < n)) ? 1 : 0;
      rank += (ek.w > key || (ek.w == key && en.w < n)) ? 1 : 0;
    }
    rank += __builtin_amdgcn_update_dpp(0, rank, 0xB1, 0xf, 0xf, true);  // quad_perm [1,0,3,2]
    rank += __builtin_amdgcn_update_dpp(0, rank, 0x4E, 0xf, 0xf, true);  // quad_perm [2,3,0,1]
    if (sub == 0 && (uint32_t)rank < need) flip_code(code32, (int)n, sgn);
  }
}

// Empties the ranking list (see k1_rank_list); with select_reset, before the first barrier.
__device__ __forceinline__ void k1_list_reset(SelectShared& sh) {
  for (int b = threadIdx.x; b < kListCap / 4; b += blockDim.x) {
    reinterpret_cast<uint4*>(sh.list_key)[b] = make_uint4(0, 0, 0, 0);
    reinterpret_cast<uint4*>(sh.list_n)[b] = make_uint4(~0u, ~0u, ~0u, ~0u);
  }
}

__device__ __forceinline__ void k1_push(SelectShared& sh, uint32_t key, int n) {
  const uint32_t slot = atomicAdd(&sh.list_count, 1u);
  sh.list_key[slot] = key;
  sh.list_n[slot] = (uint32_t)n;
}

// P[q] is element 4 * (tid + (q / 4) * T) + (q % 4) of the channel; elements past the
// channel's end hold P = 0.  All threads of the workgroup call this after the barrier that
// follows the last k1_count.
template <int NE>
__device__ __forceinline__ void k1_channel_stage(const int32_t (&P)[NE], int sgn, uint32_t need,
                                                 uint32_t* code32, SelectShared& sh) {
  static_assert(NE <= 32, "the live mask is 32 bits");
  const int T = blockDim.x, tid = threadIdx.x;
  const int32_t smask = sgn < 0 ? -1 : 0;
  auto elem = [&](int q) { return 4 * (tid + (q >> 2) * T) + (q & 3); };

  uint32_t count = 0, need_at = 0;
  const int d = k1_scan_top(sh.hist, sgn, need, need_at, count);
  if (d < 0) {  // fewer candidates of the wanted sign than flips wanted: all of them flip
#pragma unroll
    for (int q = 0; q < NE; ++q)
      if (sgn > 0 ? P[q] > 0 : P[q] < 0) flip_code(code32, elem(q), sgn);
    return;
  }
  need = need_at;
  const int32_t thr_member = d << 15, thr_flip = (d + 1) << 15;
  if (count == need && !(sgn > 0 && d == 0)) {
    // every member of the boundary bin flips (the bin that P = 0 shares needs its real count)
#pragma unroll
    for (int q = 0; q < NE; ++q)
      if ((P[q] ^ smask) >= thr_member) flip_code(code32, elem(q), sgn);
    return;
  }
  if (count <= (uint32_t)kListCap) {
    // the usual case: the boundary bin's members go straight to the ranking list
#pragma unroll
    for (int q = 0; q < NE; ++q) {
      const int32_t u = P[q] ^ smask;
      if (u >= thr_member) {
        if (u >= thr_flip) flip_code(code32, elem(q), sgn);
        else if (u > 0 || smask != 0) k1_push(sh, (uint32_t)u, elem(q));  // P = 0 is no candidate
      }
    }
    __syncthreads();
    count = sh.list_count;  // exact: without the P = 0 elements that bin 128 also counts
    k1_rank_list(sh, count, need < count ? need : count, sgn, code32);
    return;
  }
  uint32_t live = 0;
#pragma unroll
  for (int q = 0; q < NE; ++q) {
    const int32_t u = P[q] ^ smask;
    if (u >= thr_member) {
      if (u >= thr_flip) flip_code(code32, elem(q), sgn);
      else if (u > 0 || smask != 0) live |= 1u << q;  // P = 0 is no candidate
    }
  }
  if (sgn > 0 && d == 0) {  // the bin that P = 0 shares: count its real members
    __syncthreads();
    if (tid == 0) sh.wave_cnt[16] = 0;
    __syncthreads();
    if (live) atomicAdd(&sh.wave_cnt[16], (uint32_t)__popc(live));
    __syncthreads();
    count = sh.wave_cnt[16];
    if (count < need) need = count;
    if (count == 0) return;
  }

  // ---- a crowded bin: histogram passes over bits 14..7, then 7..0 of u ----
  int shift = 15;
  while (count > (uint32_t)kListCap && count != need && shift > 0) {
    shift = shift == 15 ? 7 : 0;
    __syncthreads();  // every wave has finished reading the histogram
    for (int b = tid; b < 256; b += T) sh.hist[b] = 0;
    __syncthreads();
#pragma unroll
    for (int q = 0; q < NE; ++q)
      if (live & (1u << q)) atomicAdd(&sh.hist[((uint32_t)(P[q] ^ smask) >> shift) & 255u], 1u);
    __syncthreads();
    const uint32_t d2 = scan_histogram_top(sh.hist, need, need_at, count);
    need = need_at;
#pragma unroll
    for (int q = 0; q < NE; ++q) {
      if (!(live & (1u << q))) continue;
      const uint32_t dq = ((uint32_t)(P[q] ^ smask) >> shift) & 255u;
      if (dq > d2) flip_code(code32, elem(q), sgn);
      if (dq != d2) live &= ~(1u << q);
    }
  }

  // `count` elements are still live (equal down to bit `shift`); `need` of them flip
  if (count == need) {
#pragma unroll
    for (int q = 0; q < NE; ++q)
      if (live & (1u << q)) flip_code(code32, elem(q), sgn);
    return;
  }
  if (count <= (uint32_t)kListCap) {
#pragma unroll
    for (int q = 0; q < NE; ++q)
      if (live & (1u << q)) k1_push(sh, (uint32_t)(P[q] ^ smask), elem(q));
    __syncthreads();
    k1_rank_list(sh, count, need, sgn, code32);
    return;
  }
  // more than kListCap elements equal in all their bits: the lowest indices flip.  The four
  // elements of a vector are consecutive and vectors ascend with the thread, so inside round
  // j an exclusive prefix count over the threads ranks them; the rounds follow each other.
  const int lane = tid & (kWave - 1), wid = tid / kWave;
  const int nw = (T + kWave - 1) / kWave;
  uint32_t done = 0;
  for (int round = 0; round < NE / 4; ++round) {
    const uint32_t bits = (live >> (4 * round)) & 15u;
    const uint32_t mine = (uint32_t)__popc(bits);
    const uint32_t incl = wave_prefix_sum(mine);
    __syncthreads();
    if (lane == kWave - 1) sh.wave_cnt[wid] = incl;
    __syncthreads();
    uint32_t base = done + incl - mine, total = 0;
    for (int w = 0; w < nw; ++w) {
      const uint32_t c = sh.wave_cnt[w];
      if (w < wid) base += c;
      total += c;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (bits & (1u << e)) {
        if (base < need) flip_code(code32, elem(4 * round + e), sgn);
        ++base;
      }
    done += total;
  }
}

// SQuant-E for the NV vectors of a thread: straight-line code per division method (FAST: the
// quotients through the reciprocal rs = 1/s), chosen once per workgroup by the caller.
template <int NV, bool FAST, bool WITH_P>
__device__ __forceinline__ void k1_round_all(const float (&w)[4 * NV], float s, float rs, float qmaxf,
                                             uint32_t* code32, int tid, int T, int nvec,
                                             int32_t (&P)[4 * NV], int32_t& esum) {
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    uint32_t packed = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float wv = w[4 * j + e];
      const float x = FAST ? div_by_reciprocal(wv, s, rs) : wv / s;  // the IEEE quotient either way
      const float xc = __builtin_amdgcn_fmed3f(x, -qmaxf, qmaxf);
      const float c = rintf(xc);
      packed = __builtin_amdgcn_cvt_pk_u8_f32(c + 128.0f, e, packed);
      if (WITH_P) {
        const float p = c - xc;  // exact
        P[4 * j + e] = __float_as_int(__builtin_fmaf(p, 8388608.0f, 12582912.0f)) - 0x4B400000;
        esum += P[4 * j + e];
      }
    }
    const int idx = tid + j * T;
    if (idx < nvec) code32[idx] = packed;
  }
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
  if (kChannelStage) { select_reset(sh.sel); k1_list_reset(sh.sel); }  // before the first barrier

  float amax = 0.0f;
#pragma unroll
  for (int e = 0; e < NE; e += 2) amax = fmaxf(fmaxf(amax, fabsf(w[e])), fabsf(w[e + 1]));
  amax = block_max_dpp1(amax, sh.red_f);
  const float s = amax > 0.0f ? amax / qmaxf : 1.0f;
  if (tid == 0) d.scales[m] = s;
  const bool fast = amax >= 0x1p-60f && amax <= 0x1p60f;  // uniform over the workgroup
  const float rs = 1.0f / s;

  // ---- SQuant-E (Algorithm 1): codes to LDS, perturbations kept in registers ----
  int32_t esum = 0;
  int32_t P[NE];
  if (fast) k1_round_all<NV, true, kChannelStage>(w, s, rs, qmaxf, code32, tid, T, nvec, P, esum);
  else k1_round_all<NV, false, kChannelStage>(w, s, rs, qmaxf, code32, tid, T, nvec, P, esum);

  if (kChannelStage) {
    // elements past the channel's end were loaded as 0, so their P is 0: no candidate
#pragma unroll
    for (int q = 0; q < NE; ++q) k1_count(sh.sel, P[q]);
    const int64_t ec = block_sum_dpp1(esum, sh.red_i);  // its barrier publishes codes and histogram
    const int sgn = sign_of(ec);
    const int64_t kc = flips_for(ec < 0 ? -ec : ec);
    if (kc > 0) k1_channel_stage<NE>(P, sgn, (uint32_t)(kc > N ? N : kc), code32, sh.sel);
  }
  __syncthreads();

  emit_channel(code32, nvec, d.out, m, s, a.out_format, tid, T);
}

// The variants of up to five vectors per thread are compiled for eight waves per SIMD (64
// VGPRs; the unrolled per-element code otherwise spreads over ~95): measured 8-25 % faster
// from cin = 1024 up, the extra waves hide the load latency.  Six vectors: six waves (5, 7
// and 8 measured 9-21 % slower); seven: five waves (6 is 24 % slower, 8 spills massively).
// The eight-vector variant is compiled
// for five waves per SIMD in its 256-thread form (cin up to 8192; 4 and 6 were measured
// slower), for six in its 768-thread form and keeps the 128 VGPRs that 16 waves per workgroup
// allow in its 1024-thread form.  The steps matter because whole workgroups must fit: at
// 128 VGPRs a compute unit has 16 wave slots, so workgroups of 5 to 8 waves came two at a
// time and those of 9 or more one at a time (a 2.8x cliff just above cin = 8192); at 80 VGPRs
// there are 24 slots.
template <int MAX_THREADS, int MODE, int NV>
__global__ void __launch_bounds__(MAX_THREADS)
    __attribute__((amdgpu_waves_per_eu(MAX_THREADS > 768 ? 4 : MAX_THREADS > 256 ? 6 : NV <= 5 ? 8 : NV == 6 ? 6 : 5))) squant_channel_k1(LaunchArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];  // N bytes of biased codes
  __shared__ K9Shared sh;
  int m;
  const TensorDesc d = locate(a, blockIdx.x, m);
  k1_channel<MODE, NV>(a, d, m, smem, sh);
}

// ---------------------------------------------------------------------------
// Streaming variant for channels too long for the register-resident kernel above
// (cin > 32768, e.g. the input side of a very wide fully connected layer).  Only the
// channel's codes live on chip (cin bytes of LDS); the weights are walked three times or
// more - absmax, SQuant-E with the histogram, then every step of the selection - and each
// walk recomputes the element's perturbation from the weight, which gives the same bits
// every time.  The re-reads come from the caches (one channel is a few hundred KB).
// Same selection as k1_channel_stage, with "the elements still undecided" expressed as a
// prefix of u = P or ~P instead of a per-thread bit mask.
// ---------------------------------------------------------------------------
__device__ __forceinline__ int32_t k1_round(float wv, float s, float rs, bool fast, float qmaxf,
                                            float& c) {
  const float x = fast ? div_by_reciprocal(wv, s, rs) : wv / s;  // the IEEE quotient either way
  const float xc = __builtin_amdgcn_fmed3f(x, -qmaxf, qmaxf);
  c = rintf(xc);
  const float p = c - xc;  // exact
  return __float_as_int(__builtin_fmaf(p, 8388608.0f, 12582912.0f)) - 0x4B400000;
}

// Sum of one count per thread over the workgroup (LDS counter, three barriers).
__device__ __forceinline__ uint32_t block_count(SelectShared& sh, uint32_t mine) {
  __syncthreads();
  if (threadIdx.x == 0) sh.wave_cnt[16] = 0;
  __syncthreads();
  if (mine) atomicAdd(&sh.wave_cnt[16], mine);
  __syncthreads();
  return sh.wave_cnt[16];
}

template <int MODE>
__device__ __forceinline__ void k1_stream_channel(const LaunchArgs& a, const TensorDesc& d, int m,
                                                  unsigned char* smem, K9Shared& sh) {
  constexpr bool kChannelStage = MODE == SQUANT_MODE_EKC || MODE == SQUANT_MODE_EC;
  const int T = blockDim.x, tid = threadIdx.x;
  const float qmaxf = (float)a.qmax;
  uint32_t* code32 = reinterpret_cast<uint32_t*>(smem);
  const int N = d.N, nvec = N >> 2;  // cin % 4 == 0
  const int wtype = a.wtype;
  const void* wbase = d.w;
  const size_t chan = (size_t)m * N;
  auto load4 = [&](int idx, float (&w)[4]) {
    if (wtype == SQUANT_W_F32) {
      const vf4 v = load_global_f4(static_cast<const float*>(wbase) + chan + 4 * (size_t)idx);
      w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
    } else {
      const uint32_t* p = reinterpret_cast<const uint32_t*>(static_cast<const uint16_t*>(wbase) + chan +
                                                            4 * (size_t)idx);
      const bool bf16 = wtype == SQUANT_W_BF16;
      widen_pair(load_global_u1(p), bf16, w[0], w[1]);
      widen_pair(load_global_u1(p + 1), bf16, w[2], w[3]);
    }
  };

  if (kChannelStage) { select_reset(sh.sel); k1_list_reset(sh.sel); }  // before the first barrier
  float amax = 0.0f;
  for (int idx = tid; idx < nvec; idx += T) {
    float w[4];
    load4(idx, w);
    amax = fmaxf(fmaxf(fmaxf(amax, fabsf(w[0])), fabsf(w[1])), fmaxf(fabsf(w[2]), fabsf(w[3])));
  }
  amax = block_max_dpp1(amax, sh.red_f);
  const float s = amax > 0.0f ? amax / qmaxf : 1.0f;
  if (tid == 0) d.scales[m] = s;
  const bool fast = amax >= 0x1p-60f && amax <= 0x1p60f;  // uniform over the workgroup
  const float rs = 1.0f / s;

  // ---- SQuant-E: codes to LDS, perturbations into the level-0 histogram ----
  int64_t esum = 0;
  for (int idx = tid; idx < nvec; idx += T) {
    float w[4];
    load4(idx, w);
    uint32_t packed = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float c;
      const int32_t P = k1_round(w[e], s, rs, fast, qmaxf, c);
      packed = __builtin_amdgcn_cvt_pk_u8_f32(c + 128.0f, e, packed);
      if (kChannelStage) { k1_count(sh.sel, P); esum += P; }
    }
    code32[idx] = packed;
  }

  if (kChannelStage) {
    const int64_t ec = block_sum(esum, sh.red_i);  // its barriers publish codes and histogram
    const int sgn = sign_of(ec);
    const int64_t kc = flips_for(ec < 0 ? -ec : ec);
    uint32_t need = (uint32_t)(kc > N ? N : kc);
    const int32_t smask = sgn < 0 ? -1 : 0;
    // f(u, n) for every element n of the channel, u = P (sum > 0) or ~P (sum < 0): the wanted
    // side has u > 0 resp. u >= 0, larger u is the better candidate
    auto for_each = [&](auto&& f) {
      for (int idx = tid; idx < nvec; idx += T) {
        float w[4];
        load4(idx, w);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float c;
          f(k1_round(w[e], s, rs, fast, qmaxf, c) ^ smask, 4 * idx + e);
        }
      }
    };
    auto eligible = [&](int32_t u) { return u > 0 || (smask != 0 && u == 0); };
    do {  // once; `break` leaves the selection
      if (kc <= 0) break;
      uint32_t count = 0, need_at = 0;
      const int dtop = k1_scan_top(sh.sel.hist, sgn, need, need_at, count);
      if (dtop < 0) {  // fewer candidates of the wanted sign than flips wanted: all of them flip
        for_each([&](int32_t u, int n) { if (eligible(u)) flip_code(code32, n, sgn); });
        break;
      }
      need = need_at;
      const int32_t thr_member = dtop << 15, thr_flip = (dtop + 1) << 15;
      if (sgn > 0 && dtop == 0) {  // the bin that P = 0 shares: count its real members
        uint32_t mine = 0;
        for_each([&](int32_t u, int) { mine += (u > 0 && u < thr_flip) ? 1u : 0u; });
        count = block_count(sh.sel, mine);
        if (count < need) need = count;
      }
      if (count == need) {  // everything from the boundary bin up flips
        for_each([&](int32_t u, int n) { if (u >= thr_member && eligible(u)) flip_code(code32, n, sgn); });
        break;
      }
      if (count <= (uint32_t)kListCap) {
        for_each([&](int32_t u, int n) {
          if (u >= thr_member) {
            if (u >= thr_flip) flip_code(code32, n, sgn);
            else if (eligible(u)) k1_push(sh.sel, (uint32_t)u, n);
          }
        });
        __syncthreads();
        k1_rank_list(sh.sel, count, need, sgn, code32);
        break;
      }
      // a crowded bin: flip what lies above it, then histogram passes over the lower bits.
      // Members are the eligible elements with (u >> pshift) == prefix.
      for_each([&](int32_t u, int n) { if (u >= thr_flip) flip_code(code32, n, sgn); });
      int32_t prefix = dtop;
      int pshift = 15;
      while (count > (uint32_t)kListCap && count != need && pshift > 0) {
        const int shift = pshift == 15 ? 7 : 0;
        __syncthreads();  // every wave has finished reading the histogram
        for (int b = tid; b < 256; b += T) sh.sel.hist[b] = 0;
        __syncthreads();
        for_each([&](int32_t u, int) {
          if ((u >> pshift) == prefix && eligible(u)) atomicAdd(&sh.sel.hist[((uint32_t)u >> shift) & 255u], 1u);
        });
        __syncthreads();
        const uint32_t d2 = scan_histogram_top(sh.sel.hist, need, need_at, count);
        need = need_at;
        for_each([&](int32_t u, int n) {
          if ((u >> pshift) == prefix && eligible(u) && (((uint32_t)u >> shift) & 255u) > d2)
            flip_code(code32, n, sgn);
        });
        // bits 14..7 join the prefix; the last pass (bits 7..0, bit 7 shared) pins u itself
        prefix = shift == 7 ? (prefix << 8) | (int32_t)d2 : ((prefix >> 1) << 8) | (int32_t)d2;
        pshift = shift;
      }
      if (count == need) {
        for_each([&](int32_t u, int n) {
          if ((u >> pshift) == prefix && eligible(u)) flip_code(code32, n, sgn);
        });
        break;
      }
      if (count <= (uint32_t)kListCap) {
        for_each([&](int32_t u, int n) {
          if ((u >> pshift) == prefix && eligible(u)) k1_push(sh.sel, (uint32_t)u, n);
        });
        __syncthreads();
        k1_rank_list(sh.sel, count, need, sgn, code32);
        break;
      }
      // more than kListCap elements equal in all their bits: the lowest indices flip.  Within
      // one step of the walk, element order is thread order.
      const int lane = tid & (kWave - 1), wid = tid / kWave;
      const int nw = (T + kWave - 1) / kWave;
      uint32_t done = 0;
      for (int base = 0; base < nvec && done < need; base += T) {
        const int idx = base + tid;
        uint32_t bits = 0;
        if (idx < nvec) {
          float w[4];
          load4(idx, w);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            float c;
            const int32_t u = k1_round(w[e], s, rs, fast, qmaxf, c) ^ smask;
            bits |= ((u >> pshift) == prefix && eligible(u)) ? 1u << e : 0u;
          }
        }
        const uint32_t mine = (uint32_t)__popc(bits);
        const uint32_t incl = wave_prefix_sum(mine);
        __syncthreads();
        if (lane == kWave - 1) sh.sel.wave_cnt[wid] = incl;
        __syncthreads();
        uint32_t rank = done + incl - mine, total = 0;
        for (int w2 = 0; w2 < nw; ++w2) {
          const uint32_t c = sh.sel.wave_cnt[w2];
          if (w2 < wid) rank += c;
          total += c;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (bits & (1u << e)) {
            if (rank < need) flip_code(code32, 4 * idx + e, sgn);
            ++rank;
          }
        done += total;
      }
    } while (false);
  }
  __syncthreads();

  emit_channel(code32, nvec, d.out, m, s, a.out_format, tid, T);
}

template <int MODE>
__global__ void __launch_bounds__(1024) squant_channel_k1_stream(LaunchArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];  // N bytes of biased codes
  __shared__ K9Shared sh;
  int m;
  const TensorDesc d = locate(a, blockIdx.x, m);
  k1_stream_channel<MODE>(a, d, m, smem, sh);
}

}  // namespace squant
