// SQuant-C selection for kernels that keep the per-kernel flip candidates in
// registers: a workgroup-level radix select over the candidates of one output
// channel (Algorithm 2 applied to the channel, Section 3.4; Eq. 7).
//
// Among the candidates whose sign equals the sign of the channel's accumulated
// perturbation, the `need` with the largest |v| flip, lowest kernel index first on
// ties.  Every candidate is counted into a 2 x 256-bin LDS histogram of the top 8 bits
// of |v| (one half per sign) as soon as it exists, i.e. before the channel sum and with
// it the wanted sign is known, so that ONE workgroup barrier publishes the partial
// channel sums and the histogram together.  Each wave then scans the half it needs
// (DPP prefix sums, no second barrier), which gives the digit d* holding the need-th
// largest key: everything above d* flips at once, and the few keys inside d* are ranked
// against each other through a short LDS list.  Only when that digit holds more keys
// than the list do the lower bits get histogram passes of their own; keys that are
// equal in all their bits are taken in kernel order by a workgroup prefix count.
#pragma once

#include "squant_common.h"

namespace squant {

constexpr int kListCap = 128;  // capacity of the ranking list
constexpr int kListRank = 16;  // rank through the list up to this many keys; above
                                              // it another histogram pass is cheaper than the
                                              // quadratic ranking
constexpr int kHistDummy = 512;  // bin of "no candidate"
constexpr uint32_t kNoDigit = 0xFFFFFFFFu;

struct alignas(16) SelectShared {
  uint32_t hist[528];  // [0,256): v > 0, [256,512): v < 0, 512: none; 528 = 132 x 16 bytes
  uint32_t list_count;
  uint32_t pad_[3];  // keeps the lists on 16 bytes
  uint32_t list_key[kListCap];
  uint32_t list_n[kListCap];
  uint32_t wave_cnt[17];
};

// Zeroes the histogram and the list counter; a workgroup barrier must follow before
// count_candidate.
__device__ __forceinline__ void select_reset(SelectShared& sh) {
  for (int b = threadIdx.x; b < 132; b += blockDim.x)
    reinterpret_cast<uint4*>(sh.hist)[b] = make_uint4(0, 0, 0, 0);
  if (threadIdx.x == 0) sh.list_count = 0;
}

// A candidate travels as one word: |v| (Q23, 0 < |v| < 2^23) in bits 0..22, bit 23 set when
// v < 0, and kNoCandidate (bit 24) when the kernel has none.  word >> 15 is then directly
// the histogram bin: 256 * (v < 0) + top 8 bits of |v|, or 512.
constexpr uint32_t kNoCandidate = 1u << 24;
__device__ __forceinline__ uint32_t candidate_word(int32_t v) {
  const uint32_t a = (uint32_t)(v < 0 ? -v : v);
  return v == 0 ? kNoCandidate : (a | (v < 0 ? 1u << 23 : 0u));
}

// Counts one candidate into the two-sign histogram.
__device__ __forceinline__ void count_candidate(SelectShared& sh, uint32_t word) {
  atomicAdd(&sh.hist[word >> 15], 1u);
}

// Ranking key of a channel-stage candidate: |v| if it has the sign of the channel
// sum, else 0 (not eligible).  0 < key < 2^23 for every eligible candidate.
__device__ __forceinline__ uint32_t cand_key(int32_t v, int sgn) {
  return (sgn > 0 ? v > 0 : v < 0) ? (uint32_t)(v < 0 ? -v : v) : 0u;
}

// One step against the channel sum for the code at byte `pos` of the channel's codes in
// LDS.  The codes are held biased (code + 128, 1..255), so the +-1 can be added to the
// whole dword without a carry or borrow ever leaving the byte.
__device__ __forceinline__ void flip_code(uint32_t* code32, int pos, int sgn) {
  const uint32_t delta = sgn > 0 ? 0xFFFFFFFFu : 1u;
  atomicAdd(&code32[pos >> 2], delta << ((pos & 3) * 8));
}

// Inclusive prefix sum over the 64 lanes of a wave (DPP: row_shr 1, 2, 4, 8 inside each
// row of 16, then row_bcast 15 into rows 1 and 3, row_bcast 31 into rows 2 and 3).
__device__ __forceinline__ uint32_t wave_prefix_sum(uint32_t x) {
  int v = (int)x;
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);
  return (uint32_t)v;
}

// Every wave scans 256 histogram bins from the top: finds the largest digit d* such that
// at least `need` keys have a digit >= d*.  Returns d* (kNoDigit when fewer than `need`
// keys were counted at all) and sets need_at = need - #keys above d*, count_at = hist[d*].
// Uniform over the wave; identical in every wave that reads the same histogram.
__device__ __forceinline__ uint32_t scan_histogram_top(const uint32_t* hist, uint32_t need,
                                                       uint32_t& need_at, uint32_t& count_at) {
  const int lane = threadIdx.x & (kWave - 1);
  const int first = 4 * (kWave - 1 - lane);  // lane 0 owns the four highest digits
  const uint4 h = *reinterpret_cast<const uint4*>(hist + first);  // digits first .. first+3
  const uint32_t mine = h.x + h.y + h.z + h.w;
  const uint32_t incl = wave_prefix_sum(mine);  // keys with a digit >= first
  const unsigned long long reach = __ballot(incl >= need);
  if (reach == 0ull) { need_at = 0; count_at = 0; return kNoDigit; }
  const int l = __builtin_ctzll(reach);  // first lane (highest digits) that reaches `need`
  const uint32_t above0 = (uint32_t)__builtin_amdgcn_readlane((int)(incl - mine), l);
  const uint32_t h3 = (uint32_t)__builtin_amdgcn_readlane((int)h.w, l);
  const uint32_t h2 = (uint32_t)__builtin_amdgcn_readlane((int)h.z, l);
  const uint32_t h1 = (uint32_t)__builtin_amdgcn_readlane((int)h.y, l);
  const uint32_t h0 = (uint32_t)__builtin_amdgcn_readlane((int)h.x, l);
  const uint32_t base = 4u * (uint32_t)(kWave - 1 - l);
  if (above0 + h3 >= need) { need_at = need - above0; count_at = h3; return base + 3; }
  if (above0 + h3 + h2 >= need) { need_at = need - above0 - h3; count_at = h2; return base + 2; }
  if (above0 + h3 + h2 + h1 >= need) { need_at = need - above0 - h3 - h2; count_at = h1; return base + 1; }
  need_at = need - above0 - h3 - h2 - h1;
  count_at = h0;
  return base;
}

// Every thread holds NC candidates: the candidate word cw[q], the byte offset pos[q] of the
// candidate element inside the channel's biased codes in LDS, and the kernel index nidx[q]
// that breaks ties (lowest first).  The candidates come in NC / PER_ROUND rounds: within a
// round a thread's PER_ROUND kernel indices are consecutive, ascend with q, and ascend
// from thread to thread; every index of round r is below every index of round r + 1.
// Flips the selected candidates' codes one step against the channel sum (code -= sgn).
// Must be called by all threads of the workgroup, after every candidate has been counted
// (count_candidate) and a workgroup barrier has passed.
template <int NC, int PER_ROUND>
__device__ __forceinline__ void channel_stage(const uint32_t (&cw)[NC], const int (&pos)[NC],
                                              const int (&nidx)[NC], int sgn, uint32_t need,
                                              uint32_t* code32, SelectShared& sh) {
  const uint32_t half = sgn < 0 ? 256u : 0u;
  uint32_t key[NC];
  bool live[NC];  // eligible and still undecided
  uint32_t dq[NC];
#pragma unroll
  for (int q = 0; q < NC; ++q) {
    dq[q] = (cw[q] >> 15) - half;  // top digit, < 256 exactly for the candidates of the wanted sign
    live[q] = dq[q] < 256u;
    key[q] = cw[q] & 0x7FFFFFu;
  }

  // ---- top 8 bits: already in the histogram ----
  uint32_t count = 0, need_at = 0;
  const uint32_t digit = scan_histogram_top(sh.hist + half, need, need_at, count);
  if (digit == kNoDigit) {  // fewer eligible candidates than flips wanted: all of them flip
#pragma unroll
    for (int q = 0; q < NC; ++q)
      if (live[q]) flip_code(code32, pos[q], sgn);
    return;
  }
  need = need_at;
#pragma unroll
  for (int q = 0; q < NC; ++q) {
    if (live[q] && dq[q] > digit) flip_code(code32, pos[q], sgn);
    live[q] = dq[q] == digit;
  }

  // ---- a crowded digit: histogram passes over the lower bits (from bit 7, then bit 0) ----
  int shift = 15;
  while (count > (uint32_t)kListRank && count != need && shift > 0) {
    shift = shift == 15 ? 7 : 0;
    __syncthreads();  // every wave has finished reading the histogram
    for (int b = threadIdx.x; b < 256; b += blockDim.x) sh.hist[b] = 0;
    __syncthreads();
#pragma unroll
    for (int q = 0; q < NC; ++q)
      if (live[q]) atomicAdd(&sh.hist[(key[q] >> shift) & 255u], 1u);
    __syncthreads();
    const uint32_t d2 = scan_histogram_top(sh.hist, need, need_at, count);
    need = need_at;
#pragma unroll
    for (int q = 0; q < NC; ++q) {
      if (!live[q]) continue;
      const uint32_t dq = (key[q] >> shift) & 255u;
      if (dq > d2) flip_code(code32, pos[q], sgn);
      if (dq != d2) live[q] = false;
    }
  }

  // `count` candidates are still live (same digits down to `shift`); `need` of them flip
  if (count == need) {
#pragma unroll
    for (int q = 0; q < NC; ++q)
      if (live[q]) flip_code(code32, pos[q], sgn);
    return;
  }
  if (count <= (uint32_t)kListCap) {
    // rank the live candidates against each other: larger key first, then lower kernel index
#pragma unroll
    for (int q = 0; q < NC; ++q)
      if (live[q]) {
        const uint32_t slot = atomicAdd(&sh.list_count, 1u);
        sh.list_key[slot] = key[q];
        sh.list_n[slot] = (uint32_t)nidx[q];
      }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < NC; ++q)
      if (live[q]) {
        uint32_t rank = 0;
        for (uint32_t e = 0; e < count; ++e) {
          const uint32_t ek = sh.list_key[e], en = sh.list_n[e];
          rank += (ek > key[q] || (ek == key[q] && en < (uint32_t)nidx[q])) ? 1u : 0u;
        }
        if (rank < need) flip_code(code32, pos[q], sgn);
      }
    return;
  }
  // more than kListCap keys equal in all their bits: the lowest kernel indices flip.
  // Inside a round kernel order is thread order, so an exclusive prefix count over the
  // threads ranks them; the rounds are taken one after the other.
  const int lane = threadIdx.x & (kWave - 1), wid = threadIdx.x / kWave;
  const int nw = (blockDim.x + kWave - 1) / kWave;
  uint32_t done = 0;  // live keys with a lower kernel index, counted in earlier rounds
  for (int round = 0; round < NC / PER_ROUND; ++round) {
    uint32_t mine = 0;
#pragma unroll
    for (int q = 0; q < NC; ++q)
      if (q / PER_ROUND == round) mine += live[q] ? 1u : 0u;
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
    for (int q = 0; q < NC; ++q)
      if (q / PER_ROUND == round && live[q]) {
        if (base < need) flip_code(code32, pos[q], sgn);
        ++base;
      }
    done += total;
  }
}

}  // namespace squant
