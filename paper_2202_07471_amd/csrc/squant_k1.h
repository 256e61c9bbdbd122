// SQuant kernel for 1x1 convolutions and fully connected layers (K = kh*kw = 1).
//
// With one element per kernel SQuant-K has nothing to do (k = round(|p|) = 0 for |p| <= 0.5,
// Section 3.4), every element is its own kernel, and its rounding perturbation is its
// SQuant-C candidate (Algorithm 3, "under SQuant" with k = 0).  One workgroup per output
// channel; a thread takes NV 16-byte vectors of the channel, vector j of thread t being
// vector t + j*T, so every load instruction of a wave reads 1 KB of consecutive weights.
// SQuant-E runs in registers and leaves the codes there, four to a dword (rounding by a magic
// addition leaves code + 128 in the sum's low byte, see squant_k9.h); SQuant-C is an LDS radix
// select over the signed perturbations of all cin elements of the channel that marks the
// elements to flip in a per-thread bit mask; the mask is applied to the packed codes and the
// thread writes its own vectors out, so the codes never pass through LDS and the channel
// needs no barrier after the selection.  The perturbations stay in the biased form the
// conversion leaves them in (kQ23Bias + P): sums, bins and thresholds all work on that form.
#pragma once

#include <type_traits>

#include "squant_common.h"
#include "squant_io.h"
#include "squant_k9.h"  // K9Shared, rounding constants, pack_low_bytes
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
// The routines below serve a whole workgroup on one channel (WAVE = false) or a single wave on
// a channel of its own (WAVE = true, squant_k1_wave.h): then the "threads" are the wave's lanes
// and a barrier only has to keep the compiler from moving LDS accesses across it (the LDS
// handles a wave's instructions in order).  `Sel` is SelectShared or a structure with the same
// members.
template <bool WAVE>
__device__ __forceinline__ int k1_tid() {
  if (!WAVE) return (int)threadIdx.x;
  // The wave kernel calls from inside its loop over channels.  The empty statement keeps the
  // compiler from computing everything that depends on the lane once before that loop, where
  // it does not fit the registers and comes back from scratch memory in every round.
  int lane = (int)(threadIdx.x & (kWave - 1));
  asm volatile("" : "+v"(lane));
  return lane;
}
template <bool WAVE>
__device__ __forceinline__ int k1_team() { return WAVE ? kWave : (int)blockDim.x; }
template <bool WAVE>
__device__ __forceinline__ void k1_sync() {
  if (WAVE) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  } else {
    __syncthreads();
  }
}

__device__ __forceinline__ void k1_count(SelectShared& sh, int32_t P) {
  atomicAdd(&sh.hist[(P >> 15) + 128], 1u);
}
// The same for a perturbation in biased form: bits 15..23 of kQ23Bias + P are 128 + (P >> 15)
// (the bias has 128 there and zeros below, and the bin stays within 0..256).
template <typename Sel>
__device__ __forceinline__ void k1_count_biased(Sel& sh, uint32_t pb) {
  static_assert(((kQ23Bias >> 15) & 511u) == 128u && (kQ23Bias & 0x7FFFu) == 0u, "bin taken from the biased bits");
  atomicAdd(&sh.hist[(pb >> 15) & 511u], 1u);
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

// The same ranking for the kernel that keeps its codes in registers: the lanes that rank an
// entry are not the thread that owns the element, so the list carries, in place of the index
// n = 4 * (t + j * T) + e, the word (j << 12) | (t << 2) | e, which orders the elements as n
// does and names the owner: the entries picked set bit 4 * j + e of the owner's mask, and
// after a barrier every thread reads its own.  The mask of thread t is owner_mask[t], with
// bits 32..63 (vectors 8..15) in owner_mask[T + t]; the words were zeroed before the barrier
// that precedes the pushes.  Returns the mask of this thread's
// picked elements.
constexpr int kK1MaxThreads = 1024;  // the owner word has ten bits for the thread
__device__ __forceinline__ uint32_t k1_owner_word(int tid, int q) {
  return ((uint32_t)(q >> 2) << 12) | ((uint32_t)tid << 2) | (uint32_t)(q & 3);
}
template <typename MaskT, bool WAVE = false, typename Sel>
__device__ __forceinline__ MaskT k1_rank_list_owner(Sel& sh, uint32_t* owner_mask, uint32_t count,
                                                    uint32_t need) {
  const uint32_t tid = (uint32_t)k1_tid<WAVE>(), T = (uint32_t)k1_team<WAVE>();
  const uint32_t sub = tid & 3u, groups = (count + 3u) >> 2;
  const uint4* key4 = reinterpret_cast<const uint4*>(sh.list_key);
  const uint4* n4 = reinterpret_cast<const uint4*>(sh.list_n);
  for (uint32_t i = tid >> 2; i < count; i += T >> 2) {
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
    if (sub == 0 && (uint32_t)rank < need) {
      const uint32_t j = n >> 12, t = (n >> 2) & (uint32_t)(kK1MaxThreads - 1);
      atomicOr(&owner_mask[(j >> 3) * T + t], 1u << (4u * (j & 7u) + (n & 3u)));
    }
  }
  k1_sync<WAVE>();
  MaskT mine = owner_mask[tid];
  if (sizeof(MaskT) > 4) mine |= (MaskT)owner_mask[T + tid] << (8 * sizeof(MaskT) - 32);
  return mine;
}

// Empties the ranking list (see k1_rank_list); with select_reset, before the first barrier.
template <bool WAVE = false, typename Sel>
__device__ __forceinline__ void k1_list_reset(Sel& sh) {
  for (int b = k1_tid<WAVE>(); b < kListCap / 4; b += k1_team<WAVE>()) {
    reinterpret_cast<uint4*>(sh.list_key)[b] = make_uint4(0, 0, 0, 0);
    reinterpret_cast<uint4*>(sh.list_n)[b] = make_uint4(~0u, ~0u, ~0u, ~0u);
  }
}

template <typename Sel>
__device__ __forceinline__ void k1_push(Sel& sh, uint32_t key, int n) {
  const uint32_t slot = atomicAdd(&sh.list_count, 1u);
  sh.list_key[slot] = key;
  sh.list_n[slot] = (uint32_t)n;
}

// B[q] = kQ23Bias + P of element 4 * (tid + (q / 4) * T) + (q % 4) of the channel; elements
// past the channel's end hold P = 0.  All threads of the workgroup call this after the barrier
// that follows the last k1_count_biased.  Returns the mask of this thread's elements that flip
// (bit q).  The common case costs four instructions an element: with u = P (sum > 0) or ~P
// (sum < 0), u >= thr is P >= thr resp. P <= ~thr, a compare on the biased value whose result
// is shifted into a mask.
template <int NE, typename MaskT, bool WAVE = false, typename Sel>
__device__ __forceinline__ MaskT k1_channel_stage(const uint32_t (&B)[NE], int sgn, uint32_t need,
                                                  Sel& sh, uint32_t* owner_mask) {
  static_assert(NE <= 8 * (int)sizeof(MaskT), "one mask bit per element");
  const int T = k1_team<WAVE>(), tid = k1_tid<WAVE>();
  const int32_t smask = sgn < 0 ? -1 : 0;
  auto bit = [](int q) { return (MaskT)1 << q; };
  // mask of the elements with u >= thr: a compare into the carry and an add-with-carry that
  // shifts it into the mask, as one unit so that no element needs a temporary register
  auto at_least = [&](int32_t thr) {
    MaskT all = 0;
#pragma unroll
    for (int base = (NE - 1) / 32 * 32; base >= 0; base -= 32) {  // 32 elements to a mask word
      uint32_t m = 0;
      if (sgn > 0) {
        const uint32_t t = kQ23Bias + (uint32_t)thr;  // P >= thr
#pragma unroll
        for (int q = (NE - base < 32 ? NE - base : 32) - 1; q >= 0; --q)
          asm("v_cmp_le_u32_e32 vcc, %2, %1\n\tv_addc_co_u32_e32 %0, vcc, %0, %0, vcc"
              : "+v"(m) : "v"(B[base + q]), "s"(t) : "vcc");
      } else {
        const uint32_t t = kQ23Bias + (uint32_t)~thr;  // P <= ~thr
#pragma unroll
        for (int q = (NE - base < 32 ? NE - base : 32) - 1; q >= 0; --q)
          asm("v_cmp_ge_u32_e32 vcc, %2, %1\n\tv_addc_co_u32_e32 %0, vcc, %0, %0, vcc"
              : "+v"(m) : "v"(B[base + q]), "s"(t) : "vcc");
      }
      all |= (MaskT)m << (base & (8 * (int)sizeof(MaskT) - 1));
    }
    return all;
  };

  uint32_t count = 0, need_at = 0;
  const int d = k1_scan_top(sh.hist, sgn, need, need_at, count);
  // u >= thr_flip flips outright; thr_member <= u < thr_flip is the boundary bin
  int32_t thr_flip, thr_member;
  if (d < 0) {  // fewer candidates of the wanted sign than flips wanted: all of them flip
    thr_flip = thr_member = sgn > 0 ? 1 : 0;  // P > 0 resp. ~P >= 0
  } else {
    need = need_at;
    thr_member = d << 15;
    thr_flip = (d + 1) << 15;
    // every member of the boundary bin flips (the bin that P = 0 shares needs its real count)
    if (count == need && !(sgn > 0 && d == 0)) thr_flip = thr_member;
  }
  MaskT flip = at_least(thr_flip);
  if (thr_flip == thr_member) return flip;
  MaskT live = at_least(thr_member) & ~flip;  // this thread's members of the boundary bin

  // u of element q, for the rare sides below: (B ^ m) - ((bias ^ m) - m) with m the sign mask.
  // Every phase takes the mask through a register move that the compiler cannot see through: it
  // then recomputes u where it is used instead of keeping one more register per element alive
  // across the whole selection, which does not fit.
  auto opaque = [](int32_t v) { int32_t r; asm volatile("s_mov_b32 %0, %1" : "=s"(r) : "s"(v)); return r; };
  auto u_of = [&](int q, int32_t m) { return (int32_t)((B[q] ^ (uint32_t)m) - ((kQ23Bias ^ (uint32_t)m) - (uint32_t)m)); };

  if (count <= (uint32_t)kListCap) {
    // the usual case: the boundary bin's members go straight to the ranking list
    if (live) {
      const int32_t sm = opaque(smask);
#pragma unroll
      for (int j = 0; j < NE / 4; ++j) {
        if (((uint32_t)(live >> (4 * j)) & 15u) == 0) continue;  // few vectors hold a member
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int q = 4 * j + e;
          if (live & bit(q)) {
            const int32_t u = u_of(q, sm);
            if (u > 0 || sm != 0) k1_push(sh, (uint32_t)u, k1_owner_word(tid, q));  // P = 0 is no candidate
          }
        }
      }
    }
    k1_sync<WAVE>();
    count = sh.list_count;  // exact: without the P = 0 elements that bin 128 also counts
    return flip | k1_rank_list_owner<MaskT, WAVE>(sh, owner_mask, count, need < count ? need : count);
  }

  // ---- a crowded bin: histogram passes over bits 14..7, then 7..0 of u ----
  int32_t sm = opaque(smask);
  if (sgn > 0 && d == 0) {  // the bin that P = 0 shares: drop those, count its real members
#pragma unroll
    for (int q = 0; q < NE; ++q)
      if (B[q] == kQ23Bias) live &= ~bit(q);
    k1_sync<WAVE>();
    if (tid == 0) sh.wave_cnt[16] = 0;
    k1_sync<WAVE>();
    if (live) atomicAdd(&sh.wave_cnt[16], (uint32_t)__popcll((unsigned long long)live));
    k1_sync<WAVE>();
    count = sh.wave_cnt[16];
    if (count < need) need = count;
    if (count == 0) return flip;
  }
  int shift = 15;
  while (count > (uint32_t)kListCap && count != need && shift > 0) {
    shift = shift == 15 ? 7 : 0;
    k1_sync<WAVE>();  // every wave has finished reading the histogram
    for (int b = tid; b < 256; b += T) sh.hist[b] = 0;
    k1_sync<WAVE>();
    sm = opaque(smask);
#pragma unroll
    for (int q = 0; q < NE; ++q)
      if (live & bit(q)) atomicAdd(&sh.hist[((uint32_t)u_of(q, sm) >> shift) & 255u], 1u);
    k1_sync<WAVE>();
    const uint32_t d2 = scan_histogram_top(sh.hist, need, need_at, count);
    need = need_at;
    sm = opaque(smask);
#pragma unroll
    for (int q = 0; q < NE; ++q) {
      if (!(live & bit(q))) continue;
      const uint32_t dq = ((uint32_t)u_of(q, sm) >> shift) & 255u;
      if (dq > d2) flip |= bit(q);
      if (dq != d2) live &= ~bit(q);
    }
  }

  // `count` elements are still live (equal down to bit `shift`); `need` of them flip
  if (count == need) return flip | live;
  if (count <= (uint32_t)kListCap) {
    sm = opaque(smask);
#pragma unroll
    for (int q = 0; q < NE; ++q)
      if (live & bit(q)) k1_push(sh, (uint32_t)u_of(q, sm), k1_owner_word(tid, q));
    k1_sync<WAVE>();
    return flip | k1_rank_list_owner<MaskT, WAVE>(sh, owner_mask, count, need);
  }
  // more than kListCap elements equal in all their bits: the lowest indices flip.  The four
  // elements of a vector are consecutive and vectors ascend with the thread, so inside round
  // j an exclusive prefix count over the threads ranks them; the rounds follow each other.
  const int lane = tid & (kWave - 1), wid = tid / kWave;
  const int nw = (T + kWave - 1) / kWave;
  uint32_t done = 0;
#pragma unroll 1
  for (int round = 0; round < NE / 4; ++round) {
    const uint32_t bits = (uint32_t)(live >> (4 * round)) & 15u;
    const uint32_t mine = (uint32_t)__popc(bits);
    const uint32_t incl = wave_prefix_sum(mine);
    k1_sync<WAVE>();
    if (lane == kWave - 1) sh.wave_cnt[wid] = incl;
    k1_sync<WAVE>();
    uint32_t base = done + incl - mine, total = 0;
    for (int w = 0; w < nw; ++w) {
      const uint32_t c = sh.wave_cnt[w];
      if (w < wid) base += c;
      total += c;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (bits & (1u << e)) {
        if (base < need) flip |= bit(4 * round + e);
        ++base;
      }
    done += total;
  }
  return flip;
}

// SQuant-E for the NV vectors of a thread: the packed biased codes (code + 128, four to a
// dword) and, WITH_P, the Q23 perturbations in biased form (kQ23Bias + P).  One body for every
// channel, so that the values have one home in the registers: `prescale` (uniform over the
// workgroup, almost never set) multiplies the weights by f1 * f2 first.
template <int NV, bool WITH_P>
__device__ __forceinline__ void k1_round_all(const float (&w)[4 * NV], float s, float rs, float qmaxf,
                                             bool prescale, float f1, float f2, uint32_t (&code)[NV],
                                             uint32_t (&B)[4 * NV], int32_t& esum) {
  uint32_t biased = 0;
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    // A branch that is always taken (s is finite) but that the compiler cannot fold: every
    // vector becomes a basic block of its own, which keeps the scheduler from interleaving
    // all the vectors of the thread (that costs tens of registers, and with them occupancy).
    code[j] = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) B[4 * j + e] = 0;
    if (__float_as_uint(s) + (uint32_t)j == 0xFFFFFFF0u) continue;
    float wv[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) wv[e] = w[4 * j + e];
    if (prescale) {
#pragma unroll
      for (int e = 0; e < 4; ++e) wv[e] = wv[e] * f1 * f2;
    }
    uint32_t tb[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float x = div_by_reciprocal(wv[e], s, rs);  // the IEEE quotient
      // (leaving the clamp out for the channels that do not need it, as the 3x3 kernel does, was
      // measured to cost more instructions here than the clamp itself)
      const float xc = __builtin_amdgcn_fmed3f(x, -qmaxf, qmaxf);
      const float t = xc + kRoundMagic;  // round half to even; code + 128 in the low byte
      tb[e] = __float_as_uint(t);
      if (WITH_P) {
        const float c = t - kRoundMagic;
        const float p = c - xc;  // exact
        const uint32_t pb = __float_as_uint(__builtin_fmaf(p, 8388608.0f, kQ23Magic));
        biased += pb;
        B[4 * j + e] = pb;
      }
    }
    code[j] = pack_low_bytes(tb[0], tb[1], tb[2], tb[3]);
  }
  esum = (int32_t)(biased - (uint32_t)(4 * NV) * kQ23Bias);
}

// Writes vector `idx` of output channel m (its four biased codes in c) in the requested
// format (squant_output_t): one coalesced store per thread.
__device__ __forceinline__ void k1_emit_vector(uint32_t c, int idx, void* out_base, int m, int N, float s,
                                               int format) {
  if (format == SQUANT_OUT_INT8) {
    store_global_u1(static_cast<uint8_t*>(out_base) + (size_t)m * N + 4 * (size_t)idx, c ^ 0x80808080u);
  } else if (format == SQUANT_OUT_INT4) {
    store_global_u16(static_cast<uint8_t*>(out_base) + (size_t)m * (N / 2) + 2 * (size_t)idx,
                     (uint16_t)pack_nibbles4(c));
  } else if (format == SQUANT_OUT_BF16) {
    uint16_t* out = static_cast<uint16_t*>(out_base) + (size_t)m * N + 4 * (size_t)idx;
    const vf4 v = dequant4(c, s);
    if ((reinterpret_cast<uintptr_t>(out) & 7u) == 0) {
      vu2 o;
      o.x = bf16_bits(v.x) | (bf16_bits(v.y) << 16);
      o.y = bf16_bits(v.z) | (bf16_bits(v.w) << 16);
      store_global_u2(out, o);
    } else {
      out[0] = (uint16_t)bf16_bits(v.x); out[1] = (uint16_t)bf16_bits(v.y);
      out[2] = (uint16_t)bf16_bits(v.z); out[3] = (uint16_t)bf16_bits(v.w);
    }
  } else {  // SQUANT_OUT_F32
    float* out = static_cast<float*>(out_base) + (size_t)m * N + 4 * (size_t)idx;
    const vf4 v = dequant4(c, s);
    if ((reinterpret_cast<uintptr_t>(out) & 15u) == 0) {
      store_global_f4(out, v);
    } else {
      out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
    }
  }
}

template <int MODE, int NV>
__device__ __forceinline__ void k1_channel(const LaunchArgs& a, const TensorDesc& d, int m,
                                           unsigned char* smem, K9Shared& sh) {
  constexpr bool kChannelStage = MODE == SQUANT_MODE_EKC || MODE == SQUANT_MODE_EC;
  constexpr int NE = 4 * NV;  // elements per thread
  typedef typename std::conditional<(NE > 32), uint64_t, uint32_t>::type MaskT;
  const int T = blockDim.x, tid = threadIdx.x;
  const float qmaxf = (float)a.qmax;
  uint32_t* owner_mask = reinterpret_cast<uint32_t*>(smem);  // see k1_rank_list_owner

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
  if (kChannelStage) { select_reset(sh.sel); k1_list_reset(sh.sel); owner_mask[tid] = 0; if (NE > 32) owner_mask[T + tid] = 0; }  // before the first barrier

  float amax = 0.0f;
#pragma unroll
  for (int e = 0; e < NE; e += 2) amax = fmaxf(fmaxf(amax, fabsf(w[e])), fabsf(w[e + 1]));
  amax = block_max_dpp1(amax, sh.red_f);
  const float s = amax > 0.0f ? amax / qmaxf : 1.0f;
  if (tid == 0) d.scales[m] = s;

  // ---- SQuant-E (Algorithm 1): codes and perturbations in registers ----
  // The quotients go through the reciprocal of s, which is proven exact for an absmax within
  // [2^-60, 2^60]; a channel outside is first scaled by a power of two (see squant_k9.h).
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

  if (kChannelStage) {
    // elements past the channel's end were loaded as 0, so their P is 0: no candidate.  They
    // are kept out of the histogram all the same: a wave's worth of them would land in one
    // bin, and LDS atomics on one address run one lane at a time.
#pragma unroll
    for (int j = 0; j < NV; ++j)
      if (tid + j * T < nvec) {
#pragma unroll
        for (int e = 0; e < 4; ++e) k1_count_biased(sh.sel, B[4 * j + e]);
      }
    const int64_t ec = block_sum_dpp1(esum, sh.red_i);  // its barrier publishes the histogram
    const int sgn = sign_of(ec);
    const int64_t kc = flips_for(ec < 0 ? -ec : ec);
    if (kc > 0) {
      const MaskT flip = k1_channel_stage<NE, MaskT>(B, sgn, (uint32_t)(kc > N ? N : kc), sh.sel, owner_mask);
      // one step against the channel sum for the marked elements: on the biased bytes a +-1
      // never carries into the neighbouring code
      const uint32_t sm = sgn < 0 ? ~0u : 0u;
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        const uint32_t f4 = (uint32_t)(flip >> (4 * j)) & 15u;
        const uint32_t b = (f4 * 0x204081u) & 0x01010101u;  // bit e to byte e
        code[j] -= (b ^ sm) - sm;
      }
    }
  }

  // the format is chosen once, outside the loop over the vectors
  auto emit_all = [&](int format) {
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int idx = tid + j * T;
      if (idx < nvec) k1_emit_vector(code[j], idx, d.out, m, N, s, format);
    }
  };
  if (a.out_format == SQUANT_OUT_INT8) emit_all(SQUANT_OUT_INT8);
  else if (a.out_format == SQUANT_OUT_INT4) emit_all(SQUANT_OUT_INT4);
  else if (a.out_format == SQUANT_OUT_BF16) emit_all(SQUANT_OUT_BF16);
  else emit_all(SQUANT_OUT_F32);
}

// One kernel per vector count serves every workgroup size.  Up to six vectors per thread fit
// the 64 VGPRs of eight waves per SIMD, seven and eight the 80 of six, sixteen (workgroups of
// up to 512 threads) the 128 of four.  The steps matter because
// whole workgroups must fit: at 64 VGPRs a compute unit has 32 wave slots, so two workgroups of
// 1024 threads or eight of 256 run side by side; at 80 it has 24.
template <int MODE, int NV>
__global__ void __launch_bounds__(NV <= 8 ? 1024 : 512) __attribute__((amdgpu_waves_per_eu(NV <= 6 ? 8 : NV <= 8 ? 6 : 4)))
    squant_channel_k1(LaunchArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];  // the owners' masks
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
