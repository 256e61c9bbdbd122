// SQuant-C selection for kernels that keep the per-kernel flip candidates in
// registers: a workgroup-level radix select over the candidates of one output
// channel (Algorithm 2 applied to the channel, Section 3.4; Eq. 7).
//
// Among the candidates whose sign equals the sign of the channel's accumulated
// perturbation, the `need` with the largest |v| flip, lowest kernel index first on
// ties.  One 256-bin LDS histogram of the top key digit finds the digit d* in which
// the need-th largest key lies; everything above d* flips at once, and the few
// keys inside d* are ranked against each other through a short LDS list.  Only when
// that digit holds more keys than the list does the next digit get its own
// histogram pass; keys that are equal in all their bits are taken in kernel order by a
// workgroup prefix count.
#pragma once

#include "squant_common.h"

namespace squant {

constexpr int kListCap = 128;
constexpr uint32_t kNoDigit = 0xFFFFFFFFu;

struct SelectShared {
  uint32_t hist[256];
  uint32_t bcast[4];
  uint32_t list_count;
  uint32_t list_key[kListCap];
  uint32_t list_n[kListCap];
  uint32_t wave_cnt[17];
};

// Ranking key of a channel-stage candidate: |v| if it has the sign of the channel
// sum, else 0 (not eligible).  0 < key < 2^23 for every eligible candidate.
__device__ __forceinline__ uint32_t cand_key(int32_t v, int sgn) {
  return (sgn > 0 ? v > 0 : v < 0) ? (uint32_t)(v < 0 ? -v : v) : 0u;
}

// Wave 0 scans the 256-bin histogram from the top: finds the largest digit d* such that
// at least `need` keys have a digit >= d*.  Publishes (d*, need - #keys above d*, hist[d*])
// in bcast[0..2]; d* = kNoDigit when fewer than `need` keys were counted at all.
__device__ __forceinline__ void scan_histogram(const uint32_t* hist, uint32_t need, uint32_t* bcast) {
  if (threadIdx.x < kWave) {
    const int l = threadIdx.x;
    const uint32_t h0 = hist[4 * l], h1 = hist[4 * l + 1], h2 = hist[4 * l + 2], h3 = hist[4 * l + 3];
    const uint32_t mine = h0 + h1 + h2 + h3;
    uint32_t suf = mine;  // inclusive suffix sum over lanes >= l
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
      const uint32_t o = __shfl_down(suf, off);
      if (l + off < kWave) suf += o;
    }
    const unsigned long long reach = __ballot(suf >= need);
    if (reach == 0ull) {
      if (l == 0) { bcast[0] = kNoDigit; bcast[1] = 0; bcast[2] = 0; }
    } else {
      const int top = 63 - __builtin_clzll(reach);
      if (l == top) {
        uint32_t above = suf - mine;
        uint32_t digit, cnt;
        if (above + h3 >= need) { digit = 4 * l + 3; cnt = h3; }
        else if (above + h3 + h2 >= need) { digit = 4 * l + 2; cnt = h2; above += h3; }
        else if (above + h3 + h2 + h1 >= need) { digit = 4 * l + 1; cnt = h1; above += h3 + h2; }
        else { digit = 4 * l; cnt = h0; above += h3 + h2 + h1; }
        bcast[0] = digit; bcast[1] = need - above; bcast[2] = cnt;
      }
    }
  }
}

// Every thread holds NC candidates: value v[q] (0 = none), the byte offset pos[q] of the
// candidate element inside the channel's int8 codes in LDS, and the kernel index
// n0 + q * nstride (nstride = 1: a thread owns consecutive kernels; nstride = number of
// kernel-carrying threads: thread t owns kernels t, t + nstride, ...).
// Flips the selected candidates' codes one step against the channel sum (code -= sgn).
// Must be called by all threads of the workgroup; on entry sh.list_count and sh.hist must be
// zero and a workgroup barrier must lie between their zeroing and this call.
template <int NC>
__device__ __forceinline__ void channel_stage(const int32_t (&v)[NC], const int (&pos)[NC], int n0,
                                              int nstride, int sgn, uint32_t need, int8_t* code,
                                              SelectShared& sh) {
  uint32_t key[NC];
  bool live[NC];  // still undecided
#pragma unroll
  for (int q = 0; q < NC; ++q) { key[q] = cand_key(v[q], sgn); live[q] = key[q] != 0; }

  uint32_t count = 0;
  int shift = 16;
  for (;;) {
    if (shift != 16) {  // the first pass finds the histogram already zeroed
      for (int b = threadIdx.x; b < 256; b += blockDim.x) sh.hist[b] = 0;
      __syncthreads();
    }
#pragma unroll
    for (int q = 0; q < NC; ++q)
      if (live[q]) atomicAdd(&sh.hist[(key[q] >> shift) & 255u], 1u);
    __syncthreads();
    scan_histogram(sh.hist, need, sh.bcast);
    __syncthreads();
    const uint32_t digit = sh.bcast[0];
    if (digit == kNoDigit) {  // fewer eligible candidates than flips wanted: all of them flip
#pragma unroll
      for (int q = 0; q < NC; ++q)
        if (live[q]) code[pos[q]] = (int8_t)(code[pos[q]] - sgn);
      return;
    }
    need = sh.bcast[1];
    count = sh.bcast[2];
#pragma unroll
    for (int q = 0; q < NC; ++q) {
      if (!live[q]) continue;
      const uint32_t dq = (key[q] >> shift) & 255u;
      if (dq > digit) code[pos[q]] = (int8_t)(code[pos[q]] - sgn);
      if (dq != digit) live[q] = false;
    }
    if (count <= (uint32_t)kListCap || shift == 0) break;
    shift -= 8;
    __syncthreads();  // hist and bcast are reused by the next pass
  }

  // `count` candidates are still live (same digits down to `shift`); `need` of them flip
  if (count == need) {
#pragma unroll
    for (int q = 0; q < NC; ++q)
      if (live[q]) code[pos[q]] = (int8_t)(code[pos[q]] - sgn);
    return;
  }
  if (count <= (uint32_t)kListCap) {
    // rank the live candidates against each other: larger key first, then lower kernel index
#pragma unroll
    for (int q = 0; q < NC; ++q)
      if (live[q]) {
        const uint32_t slot = atomicAdd(&sh.list_count, 1u);
        sh.list_key[slot] = key[q];
        sh.list_n[slot] = (uint32_t)(n0 + q * nstride);
      }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < NC; ++q)
      if (live[q]) {
        uint32_t rank = 0;
        for (uint32_t e = 0; e < count; ++e) {
          const uint32_t ek = sh.list_key[e], en = sh.list_n[e];
          rank += (ek > key[q] || (ek == key[q] && en < (uint32_t)(n0 + q * nstride))) ? 1u : 0u;
        }
        if (rank < need) code[pos[q]] = (int8_t)(code[pos[q]] - sgn);
      }
    return;
  }
  // more than kListCap keys equal in all their bits: the lowest kernel indices flip.
  // Kernel order is thread order within one q (nstride > 1) or thread order over all q
  // (nstride = 1), so exclusive prefix counts over the threads rank them.
  const int lane = threadIdx.x & (kWave - 1), wid = threadIdx.x / kWave;
  const int nw = (blockDim.x + kWave - 1) / kWave;
  const int rounds = nstride == 1 ? 1 : NC;
  uint32_t done = 0;  // live keys with a lower kernel index, counted in earlier rounds
  for (int round = 0; round < rounds; ++round) {
    uint32_t mine = 0;
#pragma unroll
    for (int q = 0; q < NC; ++q)
      if (nstride == 1 || q == round) mine += live[q] ? 1u : 0u;
    uint32_t incl = mine;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
      const uint32_t o = __shfl_up(incl, off);
      if (lane >= off) incl += o;
    }
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
      if ((nstride == 1 || q == round) && live[q]) {
        if (base < need) code[pos[q]] = (int8_t)(code[pos[q]] - sgn);
        ++base;
      }
    done += total;
  }
}

}  // namespace squant
