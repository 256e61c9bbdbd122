// SQuant kernel for 3x3 convolutions (K = kh*kw = 9), the bulk of a CNN's weights.
//
// One workgroup per output channel, one thread per KPT 3x3 kernels.  Nothing is staged:
// thread t reads kernels t, t+G, t+2G, ... (G = cin/KPT) straight from HBM as three 12-byte
// vectors each, so neighbouring lanes read neighbouring kernels and the three loads of a
// wave cover one contiguous 2304-byte span.  Everything up to the channel-wise decision is
// register arithmetic, written to keep the vector instruction count down (the kernel is
// bound by instruction issue as much as by memory):
//   * SQuant-E rounds by adding 1.5 * 2^23 + 128, which leaves code + 128 in the low byte of
//     the sum's bit pattern, so the nine codes of a kernel are packed into three dwords by
//     byte permutes, with no conversion;
//   * the Q23 perturbations stay biased by the bit pattern of 1.5 * 2^23: their sum is
//     corrected once, and the ranking keys are made from the biased words directly;
//   * the k <= 4 largest same-sign perturbations come out of a 25-operation three-input
//     (max3 / med3 / min3) selection network on unique keys (|p| above a 5-bit tie-break that
//     is also the shift count which turns a key into its element's flip bit);
//   * SQuant-K leaves a 9-bit flip mask per kernel; SQuant-C toggles one bit of it (flipping
//     an over-SQuant candidate back clears its bit, flipping an under-SQuant candidate sets
//     one), and the mask is applied to the packed codes once, after the channel-wise decision.
// LDS holds the two-sign histogram of SQuant-C (squant_select.h), a ranking list for the
// histogram bin the selection ends in, and finally the channel's codes for a coalesced
// 16-byte write-out; occupancy is left to the register file.
#pragma once

#include "squant_common.h"
#include "squant_io.h"
#include "squant_select.h"

namespace squant {

struct alignas(16) K9Shared {
  float red_f[16];
  int64_t red_i[16];
  SelectShared sel;
};

// Adding kRoundMagic to a clamped quotient |x| <= 127 rounds it to an integer, half to even
// (the sum lies in [2^23, 2^24), where binary32 has unit spacing, and the constant is even),
// and the sum's bit pattern ends in the byte code + 128.
constexpr float kRoundMagic = 12583040.0f;      // 1.5 * 2^23 + 128
constexpr float kQ23Magic = 12582912.0f;        // 1.5 * 2^23
constexpr uint32_t kQ23Bias = 0x4B400000u;      // its bit pattern: biased perturbation = kQ23Bias + P

// What a thread keeps of one 3x3 kernel between SQuant-K and the write-out.
struct K9Kernel {
  uint32_t d0, d1, d2;  // codes + 128: elements 0-3, 4-7, 8 (the upper bytes of d2 are not codes)
  uint32_t flips;       // bit i: element i moves one step against the sign of the kernel's sum
  uint32_t sm;          // 0 when that sign is +, ~0 when it is -
  uint32_t cand;        // the SQuant-C candidate as a candidate word (squant_select.h)
  uint32_t cand_bit;    // 1 << its element index
};

// The low bytes of four words as one dword.
__device__ __forceinline__ uint32_t pack_low_bytes(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  return __builtin_amdgcn_perm(b, a, 0x0c0c0400u) | __builtin_amdgcn_perm(d, c, 0x04000c0cu);
}

// Per-lane selects on lane masks held in scalar registers.  Written out because the compiler
// otherwise turns some of the selects below into divergent branches, which cost more than
// the one instruction and split the straight-line region the four kernels of a thread are
// scheduled in.
typedef uint64_t lanemask_t;
__device__ __forceinline__ lanemask_t lanes_uge(uint32_t a, uint32_t b) { return __builtin_amdgcn_uicmp(a, b, 35); }
__device__ __forceinline__ lanemask_t lanes_slt(int32_t a, int32_t b) { return __builtin_amdgcn_sicmp(a, b, 40); }
__device__ __forceinline__ lanemask_t lanes_sge(int32_t a, int32_t b) { return __builtin_amdgcn_sicmp(a, b, 39); }
__device__ __forceinline__ uint32_t vsel(lanemask_t m, uint32_t if_set, uint32_t if_clear) {
  uint32_t r;
  asm("v_cndmask_b32_e64 %0, %1, %2, %3" : "=v"(r) : "v"(if_clear), "v"(if_set), "s"(m));
  return r;
}

__device__ __forceinline__ uint32_t vsel0(lanemask_t m, uint32_t if_set) {  // else 0
  uint32_t r;
  asm("v_cndmask_b32_e64 %0, 0, %1, %2" : "=v"(r) : "v"(if_set), "s"(m));
  return r;
}

// SQuant-E on the nine weights w[0..8] of one kernel (Algorithm 1, rounding and element
// perturbation): packed biased codes and the nine biased Q23 perturbations.
//   FAST   take the quotients through the reciprocal rs = 1/s
//   CLAMP  clamp the quotients to [-qmax, qmax] (Section 2.2).  Only the quotient of the
//          absmax element itself can lie outside, by one rounding of s; the caller leaves the
//          clamp out for a channel whose absmax / s does not exceed qmax.
template <bool FAST, bool CLAMP = true>
__device__ __forceinline__ void k9_round(const float* w, float s, float rs, float qmaxf, K9Kernel& kk,
                                         uint32_t (&pb)[9]) {
  uint32_t tb[9];
#pragma unroll
  for (int i = 0; i < 9; ++i) {
    // x = w / s: either way the IEEE binary32 quotient
    const float x = FAST ? div_by_reciprocal(w[i], s, rs) : w[i] / s;
    const float xc = CLAMP ? __builtin_amdgcn_fmed3f(x, -qmaxf, qmaxf) : x;
    const float t = xc + kRoundMagic;
    const float c = t - kRoundMagic;  // round-half-even(xc), exact
    const float p = c - xc;           // exact
    // Q23: p * 2^23 + 1.5 * 2^23 lies in [2^23, 2^24], so the one rounding of the FMA is the
    // round-half-even of p * 2^23 and the integer sits in the low mantissa bits
    pb[i] = __float_as_uint(__builtin_fmaf(p, 8388608.0f, kQ23Magic));
    tb[i] = __float_as_uint(t);
  }
  kk.d0 = pack_low_bytes(tb[0], tb[1], tb[2], tb[3]);
  kk.d1 = pack_low_bytes(tb[4], tb[5], tb[6], tb[7]);
  kk.d2 = tb[8];
}

// SQuant-K and the perturbation update for one kernel (Algorithm 2 on the kernel,
// Algorithm 3): the flip mask, the sign, the candidate; esum += the kernel's Q23
// perturbation sum after SQuant-K; returns |sum before SQuant-K| (0: the candidate of such
// a kernel is worked out separately, see k9_recheck_kernel).
template <int MODE>
__device__ __forceinline__ uint32_t k9_flip(const uint32_t (&pb)[9], K9Kernel& kk, int32_t& esum) {
  constexpr bool kCand = MODE == SQUANT_MODE_EKC || MODE == SQUANT_MODE_EC;
  uint32_t eb = 0;
#pragma unroll
  for (int i = 0; i < 9; ++i) eb += pb[i];
  const int32_t E = (int32_t)(eb - 9u * kQ23Bias);
  const uint32_t sm = (uint32_t)(E >> 31);  // all ones when the sum is negative
  const uint32_t A = ((uint32_t)E ^ sm) - sm;  // |E|
  kk.sm = sm;

  // unique keys, larger = flips earlier.  For a positive sum (pb << 5) = base + 32 P, for a
  // negative one (~pb << 5) = base' - 32 P; the low five bits hold 31 - i.  Elements with the
  // sign of the sum are exactly those with key >= base + 32.
  uint32_t key[9];
#pragma unroll
  for (int i = 0; i < 9; ++i) key[i] = ((pb[i] ^ sm) << 5) | (uint32_t)(31 - i);
  // base' - base = (~kQ23Bias << 5) - (kQ23Bias << 5) (mod 2^32), added for a negative sum
  const uint32_t base = (kQ23Bias << 5) + (sm & (((~kQ23Bias) << 5) - (kQ23Bias << 5)));

  if (MODE == SQUANT_MODE_EC) {
    // no kernel-wise flip: k = 0, the candidate is the largest same-sign perturbation
    esum += E;
    kk.flips = 0;
    const uint32_t ck = umax3(umax3(key[0], key[1], key[2]), umax3(key[3], key[4], key[5]),
                              umax3(key[6], key[7], key[8]));
    const int32_t rel = (int32_t)(ck - base);
    kk.cand = vsel(lanes_sge(rel, 32), ((uint32_t)rel >> 5) | (sm & (1u << 23)), kNoCandidate);
    kk.cand_bit = 0x80000000u >> (ck & 31u);
    return A;
  }

  const uint32_t tt = A + (uint32_t)(kHalf - 1);  // k = tt >> 23 (an exact half rounds down)
  const int32_t r = (int32_t)(tt & 0x7FFFFFu) - (kHalf - 1);  // |sum| left after k flips, < 0: over SQuant
  esum += (int32_t)(((uint32_t)r ^ sm) - sm);

  // The three largest keys serve every kernel with k <= 2, which is all but a few in a
  // thousand; the rest of the network and of the selection runs only in waves that hold one.
  uint32_t srt[5];
  Top9Rest rest;
  top3_of_9u(key, srt, rest);
  const lanemask_t k1 = lanes_uge(tt, 1u << 23), k2 = lanes_uge(tt, 2u << 23), k3 = lanes_uge(tt, 3u << 23);
  // a key's low five bits are 31 - i, so 2^31 >> key is bit i (shift counts are taken mod 32)
  const uint32_t m0 = 0x80000000u >> (srt[0] & 31u);
  const uint32_t m1 = m0 | (0x80000000u >> (srt[1] & 31u));
  uint32_t flips = vsel(k2, m1, vsel0(k1, m0));
  uint32_t nxt = 0, thr = 0;
  if (kCand) {
    nxt = vsel(k2, srt[2], vsel(k1, srt[1], srt[0]));  // (k+1)-th largest
    thr = vsel(k2, srt[1], srt[0]);                    // k-th largest, k >= 1
  }
  if (k3 != 0) {  // uniform over the wave
    next2_of_9u(rest, srt);
    const lanemask_t k4 = lanes_uge(tt, 4u << 23);
    const uint32_t m2 = m1 | (0x80000000u >> (srt[2] & 31u));
    const uint32_t m3 = m2 | (0x80000000u >> (srt[3] & 31u));
    flips = vsel(k4, m3, vsel(k3, m2, flips));
    if (kCand) {
      nxt = vsel(k4, srt[4], vsel(k3, srt[3], nxt));
      thr = vsel(k4, srt[3], vsel(k3, srt[2], thr));
    }
  }
  kk.flips = flips;
  if (!kCand) return A;

  // ---- perturbation update (Algorithm 3): the kernel's candidate for SQuant-C ----
  const lanemask_t over = lanes_slt(r, 0);
  const uint32_t ck = vsel(over, thr, nxt);  // over: last flipped; under: first un-flipped
  const int32_t rel = (int32_t)(ck - base);         // 32 |p| + (31 - i) for a same-sign element
  const uint32_t mag = (uint32_t)rel >> 5;          // |p| of that element before any flip
  // over: the post-flip value kOne - mag with the sign opposite to the sum; under: mag with
  // the sign of the sum
  const uint32_t sbit = sm & (1u << 23);
  const uint32_t word = vsel(over, ((2u << 23) - sbit) - mag, mag | sbit);
  kk.cand = vsel(lanes_sge(rel, 32), word, kNoCandidate);
  kk.cand_bit = 0x80000000u >> (ck & 31u);
  return A;
}

// Moves the elements named by the flip mask one step against the kernel's sign: on the
// biased bytes a +-1 never carries into the neighbouring code.
__device__ __forceinline__ void k9_apply_flips(K9Kernel& kk) {
  uint32_t b0, b1, b2;
  spread_flip_bits(kk.flips, b0, b1, b2);
  kk.d0 -= (b0 ^ kk.sm) - kk.sm;
  kk.d1 -= (b1 ^ kk.sm) - kk.sm;
  kk.d2 -= (b2 ^ kk.sm) - kk.sm;
}

// Cold path (a rolled loop) for a thread that saw a kernel whose perturbation sum is exactly zero.  Nothing
// is masked in such a kernel: its candidate is the largest |p| of either sign, lowest index
// first.  It has k = 0, so its perturbations are those of plain rounding and are recomputed
// here from the weights in memory; returns (sum is zero, candidate perturbation, element index).
__device__ __forceinline__ int3 k9_recheck_kernel(const void* w, size_t first, int wtype, float s, float qmaxf) {
  int32_t best = 0, bv = 0, sum = 0;
  int bi = 0;
#pragma unroll 1
  for (int i = 0; i < 9; ++i) {
    float x = load_weight(w, first + i, wtype) / s;
    x = fminf(fmaxf(x, -qmaxf), qmaxf);
    const float p = rintf(x) - x;
    const int32_t P = __float2int_rn(p * 8388608.0f);
    const int32_t ap = P < 0 ? -P : P;
    sum += P;
    if (ap > best) { best = ap; bv = P; bi = i; }
  }
  return make_int3(sum == 0 ? 1 : 0, bv, bi);
}

// The candidate of a zero-sum kernel into the kernel's record: flipping it moves the element
// against its own sign, so that sign becomes the kernel's (the flip mask is empty, so the
// sign has had no other use).
__device__ __forceinline__ void k9_set_zero_sum_candidate(K9Kernel& kk, int32_t v, int index) {
  kk.cand = candidate_word(v);
  kk.cand_bit = 1u << index;
  kk.sm = v < 0 ? ~0u : 0u;
}

// Kernel q of a thread: nine floats at `base` (uniform, the channel's kernels q*G ...)
// plus the lane's element offset, as three 12-byte loads, into w[9q .. 9q+8].
template <int NW>
__device__ __forceinline__ void k9_load_kernel(float (&w)[NW], int q, const float* base,
                                               uint32_t lane_off) {
#pragma unroll
  for (int j = 0; j < 3; ++j) {
    const vf3 v = load_global_f3(base + (lane_off + 3 * j));
    w[9 * q + 3 * j] = v.x; w[9 * q + 3 * j + 1] = v.y; w[9 * q + 3 * j + 2] = v.z;
  }
}

// The same for 16-bit weights (binary16 or bfloat16).  Kernel n starts at half-word 9n of
// the channel, which is dword aligned for even n only, so five aligned dwords starting at
// half-word 9n - (n & 1) are read and shifted down by one half-word for odd n.  chan32 is the
// channel's first dword (the channel has 9 * cin half-words, cin % 4 == 0, so it is dword
// aligned and ends with the last kernel's last half-word: no load reaches past it).
template <int NW>
__device__ __forceinline__ void k9_load_kernel16(float (&w)[NW], int q, const uint32_t* chan32,
                                                 uint32_t n, bool bf16) {
  const uint32_t h0 = 9u * n;
  const uint32_t sh = (h0 & 1u) << 4;
  const uint32_t* p = chan32 + (h0 >> 1);
  uint32_t d[5];
#pragma unroll
  for (int j = 0; j < 5; ++j) d[j] = load_global_u1(p + j);
  uint32_t u[5];
#pragma unroll
  for (int j = 0; j < 4; ++j) u[j] = __builtin_amdgcn_alignbit(d[j + 1], d[j], sh);
  u[4] = d[4] >> sh;
#pragma unroll
  for (int j = 0; j < 4; ++j) widen_pair(u[j], bf16, w[9 * q + 2 * j], w[9 * q + 2 * j + 1]);
  float unused;
  widen_pair(u[4], bf16, w[9 * q + 8], unused);
}

// Sum over the wave of values with |v| <= 2^25 (the 16 lanes of a row add up to at most 2^29).
__device__ __forceinline__ int64_t wave_sum_rows(int32_t v) {
  v += dpp_i32<0xB1>(v);
  v += dpp_i32<0x4E>(v);
  v += dpp_i32<0x141>(v);
  v += dpp_i32<0x140>(v);
  return (int64_t)__builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) +
         __builtin_amdgcn_readlane(v, 32) + __builtin_amdgcn_readlane(v, 48);
}

// Workgroup-wide maximum / sum with the number of waves known at compile time (NWC = 0: taken
// from the launch).  One barrier each (none for a one-wave workgroup), for callers that pass
// another barrier before they use the same slots again.
template <int NWC>
__device__ __forceinline__ float k9_block_max(float v, float* slot) {
  if (NWC == 0) return block_max_dpp1(v, slot);
  v = wave_max_dpp(v);
  if (NWC == 1) return v;
  if ((threadIdx.x & (kWave - 1)) == 0) slot[threadIdx.x / kWave] = v;
  __syncthreads();
  float r = slot[0];
#pragma unroll
  for (int i = 1; i < NWC; ++i) r = fmaxf(r, slot[i]);
  return r;
}
template <int NWC>
__device__ __forceinline__ int64_t k9_block_sum(int64_t ws, int64_t* slot) {
  if (NWC == 1) return ws;
  const int nw = NWC ? NWC : (int)((blockDim.x + kWave - 1) / kWave);
  if ((threadIdx.x & (kWave - 1)) == 0) slot[threadIdx.x / kWave] = ws;
  __syncthreads();
  int64_t r = slot[0];
  if (NWC) {
#pragma unroll
    for (int i = 1; i < NWC; ++i) r += slot[i];
  } else {
    for (int i = 1; i < nw; ++i) r += slot[i];
  }
  return r;
}
// Zeroes the histogram and the list counter (132 sixteen-byte stores and one more).
template <int NWC>
__device__ __forceinline__ void k9_select_reset(SelectShared& sel) {
  if (NWC == 0) { select_reset(sel); return; }
#pragma unroll
  for (int b = 0; b < 132; b += kWave * NWC)
    if (b + (int)threadIdx.x < 132) reinterpret_cast<uint4*>(sel.hist)[b + threadIdx.x] = make_uint4(0, 0, 0, 0);
  if (threadIdx.x == 0) sel.list_count = 0;
}

// SQuant-C on the kernels a thread holds (Algorithm 2 applied to the channel; Eq. 7): among
// the candidates with the sign of the channel sum `ec`, the round(|ec|) with the largest |v|
// (lowest kernel index first on ties) get their flip-mask bit toggled.  Every candidate has
// been counted into the two-sign histogram and a workgroup barrier has passed.  `list` is
// LDS room for one dword per kernel of the channel (the place the codes go afterwards).
// Uniform control flow: every wave scans the histogram for itself and reaches the same
// decisions.
template <int KPT>
__device__ __forceinline__ void k9_channel_flip(K9Kernel (&kk)[KPT], int64_t ec, int N, int t, int G,
                                                bool active, uint32_t* list, SelectShared& sel) {
  const int64_t a = ec < 0 ? -ec : ec;
  int64_t kc = flips_for(a);
  if (kc <= 0) return;
  if (kc > N) kc = N;
  const uint32_t side = ec < 0 ? 256u : 0u;  // histogram half of the wanted sign
  uint32_t need_at = 0, count_at = 0;
  const uint32_t digit = scan_histogram_top(sel.hist + side, (uint32_t)kc, need_at, count_at);
  // candidates of the wanted sign have bins side .. side + 255; those above bin `lo` flip
  // at once; when fewer candidates exist than flips are wanted (no digit) all of them flip,
  // and so do all those of bin `digit` when the count there is exactly what is still wanted
  uint32_t lo;
  bool rank = false;  // only some of the candidates in bin `lo` flip
  if (digit == kNoDigit) lo = side - 1u;
  else if (count_at == need_at) lo = side + digit - 1u;
  else { lo = side + digit; rank = true; }
  const uint32_t span = side + 255u - lo;
  bool at[KPT];
#pragma unroll
  for (int q = 0; q < KPT; ++q) {
    const uint32_t bin = kk[q].cand >> 15;
    const bool above = bin - lo - 1u < span;
    at[q] = rank && active && bin == lo;
    if (above && active) kk[q].flips ^= kk[q].cand_bit;
  }
  if (!rank) return;
  // Rank the candidates of bin `lo` among themselves: they agree in the top eight bits of
  // |v|, so the low fifteen above "4095 - kernel index" order them (cin <= 4096).
  uint32_t comp[KPT];
#pragma unroll
  for (int q = 0; q < KPT; ++q) {
    comp[q] = ((kk[q].cand & 0x7FFFu) << 12) | (uint32_t)(4095 - (t + q * G));
    if (at[q]) list[atomicAdd(&sel.list_count, 1u)] = comp[q];
  }
  bool any = false;
#pragma unroll
  for (int q = 0; q < KPT; ++q) any |= at[q];
  __syncthreads();
  if (__ballot(any) != 0ull) {
    uint32_t above[KPT];
#pragma unroll
    for (int q = 0; q < KPT; ++q) above[q] = 0;
    for (uint32_t e = 0; e < count_at; ++e) {
      const uint32_t other = list[e];
#pragma unroll
      for (int q = 0; q < KPT; ++q) above[q] += other > comp[q] ? 1u : 0u;
    }
#pragma unroll
    for (int q = 0; q < KPT; ++q)
      if (at[q] && above[q] < need_at) kk[q].flips ^= kk[q].cand_bit;
  }
  __syncthreads();  // the list's place is about to take the codes
}

// SQuant-E and SQuant-K on all the kernels of a thread.
//   PRESCALE  the weights are first multiplied by the powers of two f1 and f2 (and s, rs are
//             those of the scaled channel): see k9_channel
template <int MODE, int KPT, bool PRESCALE, bool CLAMP>
__device__ __forceinline__ void k9_solve_all(const float (&w)[9 * KPT], float s, float rs, float qmaxf,
                                             float f1, float f2, K9Kernel (&kk)[KPT], int32_t& esum,
                                             uint32_t& amin) {
#pragma unroll
  for (int q = 0; q < KPT; ++q) {
    // A branch that is always taken (s is finite) but that the compiler cannot fold: it makes
    // every kernel a basic block of its own, which keeps the scheduler from interleaving the
    // kernels (that costs 118 instead of about 90 registers) at the price of two scalar
    // instructions.
    kk[q].d0 = kk[q].d1 = kk[q].d2 = kk[q].flips = kk[q].sm = kk[q].cand_bit = 0;
    kk[q].cand = kNoCandidate;
    if (__float_as_uint(s) + (uint32_t)q == 0xFFFFFFF0u) continue;
    float x[9];
#pragma unroll
    for (int i = 0; i < 9; ++i) {
      x[i] = PRESCALE ? w[9 * q + i] * f1 * f2 : w[9 * q + i];
    }
    uint32_t pb[9];
    k9_round<true, CLAMP>(x, s, rs, qmaxf, kk[q], pb);
    if (MODE != SQUANT_MODE_E) {
      amin = umin2(amin, k9_flip<MODE>(pb, kk[q], esum));
      if (MODE == SQUANT_MODE_EK) k9_apply_flips(kk[q]);
    }
  }
}

// One workgroup per output channel.  Thread t owns the KPT 3x3 kernels t, t + G, t + 2G, ...
// (G = cin / KPT); KPT is 4 for wide layers and 2 or 1 for narrow ones, so that the waves
// stay full.
//   WT   the weight type when it is known at compile time (squant_wtype_t), -1: the launch's
//   NWC  the waves per workgroup when known at compile time, 0: the launch's
template <int MODE, int KPT, int WT = -1, int NWC = 0>
__device__ __forceinline__ void k9_channel(const LaunchArgs& a, const TensorDesc& d, int m,
                                           unsigned char* smem, K9Shared& sh) {
  constexpr bool kChannelStage = MODE == SQUANT_MODE_EKC || MODE == SQUANT_MODE_EC;
  const int T = NWC ? NWC * kWave : (int)blockDim.x, tid = threadIdx.x;
  const int wtype = WT >= 0 ? WT : a.wtype;
  const float qmaxf = (float)a.qmax;
  uint8_t* code8 = reinterpret_cast<uint8_t*>(smem);  // biased codes: code + 128

  const int N = d.N, G = N / KPT;
  const int L = 9 * N, nvec = L >> 2;  // dwords of codes (cin % 4 == 0)
  const bool active = tid < G;
  const int t = active ? tid : 0;  // idle threads shadow thread 0's loads and write nothing
  float w[9 * KPT];
  if (wtype == SQUANT_W_F32) {
    const float* src = static_cast<const float*>(d.w) + (size_t)m * L;
#pragma unroll
    for (int q = 0; q < KPT; ++q) k9_load_kernel(w, q, src + (size_t)q * (9 * G), 9u * (uint32_t)t);
  } else {
    const uint32_t* chan32 =
        reinterpret_cast<const uint32_t*>(static_cast<const uint16_t*>(d.w) + (size_t)m * L);
    const bool bf16 = wtype == SQUANT_W_BF16;
#pragma unroll
    for (int q = 0; q < KPT; ++q) k9_load_kernel16(w, q, chan32, (uint32_t)(t + q * G), bf16);
  }
  if (kChannelStage) k9_select_reset<NWC>(sh.sel);  // before the first barrier

  float amax = 0.0f;
#pragma unroll
  for (int j = 0; j + 1 < 9 * KPT; j += 2) amax = fmaxf(fmaxf(amax, fabsf(w[j])), fabsf(w[j + 1]));
  if ((9 * KPT) & 1) amax = fmaxf(amax, fabsf(w[9 * KPT - 1]));
  amax = k9_block_max<NWC>(amax, sh.red_f);
  const float s = amax > 0.0f ? amax / qmaxf : 1.0f;
  if (tid == 0) d.scales[m] = s;

  K9Kernel kk[KPT];
  int32_t esum = 0;
  uint32_t amin = ~0u;  // smallest |kernel sum| of this thread: 0 flags an exact-zero kernel
  // The quotients w / s go through the reciprocal of s, which is proven exact while nothing
  // under- or overflows on the way: absmax within [2^-60, 2^60].  A channel outside that range
  // is first scaled by a power of two, weights and scale alike (exact, and the quotients are
  // those of the unscaled channel; an element that leaves the normal range on the way down is
  // more than 2^60 below the absmax and rounds to code 0 with perturbation 0 either way).
  // One uniform branch around all the kernels of the thread, each side one straight-line region.
  if (amax <= 0x1p60f && (amax >= 0x1p-60f || amax == 0.0f)) {
    const float rs = 1.0f / s;
    // the largest quotient of the channel: no element needs the clamp unless this one does
    if (div_by_reciprocal(amax, s, rs) <= qmaxf) k9_solve_all<MODE, KPT, false, false>(w, s, rs, qmaxf, 1.0f, 1.0f, kk, esum, amin);
    else k9_solve_all<MODE, KPT, false, true>(w, s, rs, qmaxf, 1.0f, 1.0f, kk, esum, amin);
  } else {
    const float f1 = amax < 1.0f ? 0x1p64f : 0x1p-64f;
    const float a1 = amax * f1;
    const float f2 = a1 < 0x1p-60f ? 0x1p64f : a1 > 0x1p60f ? 0x1p-64f : 1.0f;
    const float s2 = s * f1 * f2;
    k9_solve_all<MODE, KPT, true, true>(w, s2, 1.0f / s2, qmaxf, f1, f2, kk, esum, amin);
  }

  if (kChannelStage) {
    if (amin == 0u && active) {
#pragma unroll
      for (int q = 0; q < KPT; ++q) {
        const int3 z = k9_recheck_kernel(d.w, (size_t)m * L + 9 * (t + q * G), wtype, s, qmaxf);
        if (z.x) k9_set_zero_sum_candidate(kk[q], z.y, z.z);
      }
    }
    // candidates into the histogram before the wanted sign is known: one barrier then
    // publishes the partial sums and the histogram
    if (active) {
#pragma unroll
      for (int q = 0; q < KPT; ++q) count_candidate(sh.sel, kk[q].cand);
    }
    // after SQuant-K a kernel's sum is at most a half; without it (mode E&C) up to 4.5
    const int64_t ws = MODE == SQUANT_MODE_EC ? wave_sum_dpp(active ? esum : 0)
                                              : wave_sum_rows(active ? esum : 0);
    const int64_t ec = k9_block_sum<NWC>(ws, sh.red_i);
    k9_channel_flip<KPT>(kk, ec, N, t, G, active, reinterpret_cast<uint32_t*>(smem), sh.sel);
#pragma unroll
    for (int q = 0; q < KPT; ++q) k9_apply_flips(kk[q]);
  }

  if (active) {
#pragma unroll
    for (int q = 0; q < KPT; ++q) {
      uint8_t* dst = code8 + 9 * (t + q * G);
      const uint64_t lo = (uint64_t)kk[q].d0 | ((uint64_t)kk[q].d1 << 32);
      __builtin_memcpy(dst, &lo, 8);
      dst[8] = (uint8_t)kk[q].d2;
    }
  }
  __syncthreads();

  emit_channel(reinterpret_cast<const uint32_t*>(smem), nvec, d.out, m, s, a.out_format, tid, T);
}

// Compiled for five waves per SIMD (at most 102 VGPRs): left alone, the scheduler interleaves
// the four kernels of a thread further than the register file pays for.
template <int MAX_THREADS, int MODE, int KPT, int WT = -1, int NWC = 0>
__global__ void __launch_bounds__(MAX_THREADS) __attribute__((amdgpu_waves_per_eu(5)))
    squant_channel_k9(LaunchArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];  // 9*N bytes of codes
  __shared__ K9Shared sh;
  int m;
  const TensorDesc d = locate(a, blockIdx.x, m);
  k9_channel<MODE, KPT, WT, NWC>(a, d, m, smem, sh);
}

// ---------------------------------------------------------------------------
// Depthwise 3x3 convolutions (cin per group = 1): an output channel is a single 3x3 kernel,
// so one thread takes a whole channel - its own absmax scale, SQuant-E and SQuant-K in
// registers through the same routines.  SQuant-C on a one-kernel channel: after SQuant-K the
// channel's sum is the kernel's, at most 0.5, so nothing flips (E&K&C equals E&K); without
// SQuant-K (mode E&C) the kernel's one candidate flips when the sum rounds to 1 or more.
// `item` is the workgroup's index within the tensor: thread t has channel item * T + t.
// No workgroup-wide step, no LDS.
// ---------------------------------------------------------------------------
template <int MODE>
__device__ __forceinline__ void dw9_channels(const LaunchArgs& a, const TensorDesc& d, int item) {
  constexpr int KM = MODE == SQUANT_MODE_EKC ? SQUANT_MODE_EK : MODE;
  const int c = item * (int)blockDim.x + (int)threadIdx.x;
  if (c >= d.M) return;
  const float qmaxf = (float)a.qmax;
  float w[9];
  if (a.wtype == SQUANT_W_F32) {
    k9_load_kernel(w, 0, static_cast<const float*>(d.w), 9u * (uint32_t)c);
  } else {
#pragma unroll
    for (int i = 0; i < 9; ++i) w[i] = load_weight(d.w, 9 * (size_t)c + i, a.wtype);
  }
  float amax = 0.0f;
#pragma unroll
  for (int i = 0; i < 9; ++i) amax = fmaxf(amax, fabsf(w[i]));
  const float s = amax > 0.0f ? amax / qmaxf : 1.0f;
  d.scales[c] = s;

  K9Kernel kk;
  uint32_t pb[9];
  k9_round<false>(w, s, 0.0f, qmaxf, kk, pb);
  if (MODE != SQUANT_MODE_E) {
    int32_t esum = 0;
    k9_flip<KM>(pb, kk, esum);
    if (MODE == SQUANT_MODE_EC) {
      // the channel is this kernel: its candidate has the sign of the sum (none if the sum is 0)
      const int32_t mag = esum < 0 ? -esum : esum;
      if (flips_for(mag) >= 1 && kk.cand != kNoCandidate) kk.flips ^= kk.cand_bit;
    }
    k9_apply_flips(kk);
  }

  int code[9];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    code[i] = (int)((kk.d0 >> (8 * i)) & 255u) - 128;
    code[4 + i] = (int)((kk.d1 >> (8 * i)) & 255u) - 128;
  }
  code[8] = (int)(kk.d2 & 255u) - 128;
  if (a.out_format == SQUANT_OUT_INT8) {
    int8_t* out = static_cast<int8_t*>(d.out) + 9 * (size_t)c;
#pragma unroll
    for (int i = 0; i < 9; ++i) out[i] = (int8_t)code[i];
  } else if (a.out_format == SQUANT_OUT_INT4) {
    uint8_t* out = static_cast<uint8_t*>(d.out) + 5 * (size_t)c;  // rows of (9 + 1) / 2 bytes
#pragma unroll
    for (int j = 0; j < 5; ++j) {
      const uint32_t lo = (uint32_t)code[2 * j] & 0xFu;
      const uint32_t hi = j < 4 ? ((uint32_t)code[2 * j + 1] & 0xFu) : 0u;
      out[j] = (uint8_t)(lo | (hi << 4));
    }
  } else if (a.out_format == SQUANT_OUT_BF16) {
    uint16_t* out = static_cast<uint16_t*>(d.out) + 9 * (size_t)c;
#pragma unroll
    for (int i = 0; i < 9; ++i) out[i] = (uint16_t)bf16_bits((float)code[i] * s);
  } else {  // SQUANT_OUT_F32
    float* out = static_cast<float*>(d.out) + 9 * (size_t)c;
#pragma unroll
    for (int i = 0; i < 9; ++i) out[i] = (float)code[i] * s;
  }
}

template <int MODE>
__global__ void __launch_bounds__(256) squant_channel_dw9(LaunchArgs a) {
  int m;
  const TensorDesc d = locate(a, blockIdx.x, m);
  dw9_channels<MODE>(a, d, m);
}

}  // namespace squant
