// Streaming SQuant kernel: the fallback for output channels that fit none of the kernels
// which hold a channel on chip (a 3x3 layer beyond cin 4096, any other kernel size beyond
// what LDS holds, very long or unaligned 1x1 / FC rows).  Any cin, kh*kw, alignment, weight
// type and output format; no memory beyond the inputs, the outputs and a few KB of LDS.
//
// One workgroup per output channel.  Nothing about the channel is kept between steps:
// every step walks the weights again (they come from the caches after the first walk) and
// recomputes what it needs, which gives the same bits every time.
//   1. absmax walk -> scale (Section 4, per-channel range)
//   2. per kernel (one thread per kernel): SQuant-E and SQuant-K (Algorithm 1, Algorithm 2)
//      as a sum walk followed by k + 1 arg-max walks over the kernel's elements, which yield
//      the k-th largest same-sign key (the flip threshold) and the Algorithm 3 candidate;
//      the kernel's sum goes into the channel sum, its candidate into a two-sign histogram
//   3. SQuant-C (Algorithm 2 on the channel, Eq. 7): the kernels are ranked by the composite
//      key (|v| << 32) | ~index, which is unique, so "the k_c largest, lowest index first on
//      ties" is "composite >= C*".  C* comes from a radix select: the histogram of step 2
//      gives the top eight bits; while the bin the selection ends in holds more than 128
//      members another walk counts the next eight bits, otherwise one walk collects the
//      members into an LDS list that is ranked directly
//   4. final walk: every kernel is solved once more, its flips and (if its composite reaches
//      C*) its candidate's flip are applied, and the output is written in its final format.
#pragma once

#include "squant_common.h"
#include "squant_io.h"
#include "squant_select.h"

namespace squant {

constexpr int kStreamThreads = 1024;
constexpr int kStreamListCap = 128;

struct alignas(16) StreamShared {
  float red_f[16];
  int64_t red_i[16];
  uint32_t hist[528];  // [0,256): v > 0, [256,512): v < 0, 512: no candidate
  uint64_t list[kStreamListCap];
  uint64_t result;
  uint32_t list_count;
};

struct StreamChannel {
  const void* w;   // tensor base
  size_t first;    // index of the channel's first element
  int wtype;
  float s, rs, qmaxf;
  bool fast;       // quotients through the reciprocal (absmax within its proven range)
};

// SQuant-E on one weight: code and Q23 perturbation.
__device__ __forceinline__ int32_t st_round(const StreamChannel& ch, size_t e, int& code) {
  const float wv = load_weight(ch.w, ch.first + e, ch.wtype);
  const float x = ch.fast ? div_by_reciprocal(wv, ch.s, ch.rs) : wv / ch.s;  // the IEEE quotient either way
  const float xc = fminf(fmaxf(x, -ch.qmaxf), ch.qmaxf);
  const float c = rintf(xc);
  code = (int)c;
  return __float2int_rn((c - xc) * 8388608.0f);  // c - xc is exact
}

// Unique ranking key of element i with perturbation magnitude a > 0: larger |p| first, then
// lower index.
__device__ __forceinline__ uint64_t st_key(uint32_t a, uint32_t i) { return ((uint64_t)a << 32) | (uint32_t)~i; }

struct StreamKernel {
  int64_t sum_after;  // the kernel's Q23 perturbation sum after SQuant-K
  uint64_t thr;       // elements with the kernel's sign and key >= thr flip (~0: none)
  int32_t sgn;        // sign of the sum before SQuant-K
  int32_t cand_i;     // Algorithm 3 candidate: element index, -1 = none
  int32_t cand_v;     // its Q23 perturbation (after its SQuant-K flip, if it had one)
};

// SQuant-K and the perturbation update for kernel n (K elements from element n * K).
template <int MODE>
__device__ StreamKernel st_solve_kernel(const StreamChannel& ch, size_t n, int K) {
  const size_t e0 = n * (size_t)K;
  StreamKernel r;
  r.thr = ~0ull;
  r.cand_i = -1;
  r.cand_v = 0;
  int64_t E = 0;
  for (int i = 0; i < K; ++i) {
    int code;
    E += st_round(ch, e0 + i, code);
  }
  r.sgn = E > 0 ? 1 : E < 0 ? -1 : 0;
  r.sum_after = E;
  if (MODE == SQUANT_MODE_E) return r;
  const int64_t A = E < 0 ? -E : E;
  const int64_t k = MODE == SQUANT_MODE_EC ? 0 : flips_for(A);
  if (r.sgn == 0) {
    // nothing is masked: the largest |p| of either sign, lowest index first
    uint64_t best = 0;
    int32_t bv = 0;
    for (int i = 0; i < K; ++i) {
      int code;
      const int32_t P = st_round(ch, e0 + i, code);
      const uint64_t key = st_key((uint32_t)(P < 0 ? -P : P), (uint32_t)i);
      if (P != 0 && key > best) { best = key; bv = P; }
    }
    if (best) { r.cand_i = (int32_t)~(uint32_t)best; r.cand_v = bv; }
    return r;
  }
  // the k + 1 largest keys among the elements with the sign of the sum, one walk each
  uint64_t last = ~0ull, kth = 0, nxt = 0;
  for (int64_t round = 0; round <= k; ++round) {
    uint64_t best = 0;
    for (int i = 0; i < K; ++i) {
      int code;
      const int32_t P = st_round(ch, e0 + i, code);
      const int32_t a = r.sgn > 0 ? P : -P;
      if (a <= 0) continue;
      const uint64_t key = st_key((uint32_t)a, (uint32_t)i);
      if (key < last && key > best) best = key;
    }
    if (best == 0) break;  // no further element of that sign
    last = best;
    if (round == k - 1) kth = best;
    if (round == k) nxt = best;
  }
  if (k >= 1) r.thr = kth;  // exists: Appendix B.1
  r.sum_after = E - (int64_t)r.sgn * k * kOne;
  if (k * (int64_t)kOne > A) {  // over SQuant: the last flipped element, post-flip value
    r.cand_i = (int32_t)~(uint32_t)kth;
    r.cand_v = r.sgn * ((int32_t)(kth >> 32) - kOne);
  } else if (nxt) {             // under SQuant: the first un-flipped element of that sign
    r.cand_i = (int32_t)~(uint32_t)nxt;
    r.cand_v = r.sgn * (int32_t)(nxt >> 32);
  }
  return r;
}

// Counts a candidate perturbation into the two-sign histogram (bin 512: no candidate).
__device__ __forceinline__ void count_candidate_bin(uint32_t* hist, int32_t v) {
  const uint32_t a = (uint32_t)(v < 0 ? -v : v);
  atomicAdd(&hist[v == 0 ? 512u : (v < 0 ? 256u : 0u) + (a >> 15)], 1u);
}

// Composite ranking key of kernel n's candidate for SQuant-C, 0 when it is not eligible.
__device__ __forceinline__ uint64_t st_composite(int32_t v, int sgn_c, size_t n) {
  if (v == 0 || (v > 0) != (sgn_c > 0)) return 0;
  return ((uint64_t)(uint32_t)(v < 0 ? -v : v) << 32) | (uint32_t)~(uint32_t)n;
}

template <int MODE>
__device__ void stream_channel(const LaunchArgs& a, const TensorDesc& d, int m, StreamShared& sh) {
  constexpr bool kChannelStage = MODE == SQUANT_MODE_EKC || MODE == SQUANT_MODE_EC;
  const int T = blockDim.x, tid = threadIdx.x;
  const int K = d.K;
  const size_t N = (size_t)d.N, L = N * (size_t)K;
  StreamChannel ch;
  ch.w = d.w;
  ch.first = (size_t)m * L;
  ch.wtype = a.wtype;
  ch.qmaxf = (float)a.qmax;

  for (int b = tid; b < 528; b += T) sh.hist[b] = 0;
  if (tid == 0) sh.list_count = 0;
  float amax = 0.0f;
  for (size_t e = tid; e < L; e += T) amax = fmaxf(amax, fabsf(load_weight(ch.w, ch.first + e, ch.wtype)));
  amax = block_max_dpp1(amax, sh.red_f);  // its barrier also publishes the cleared histogram
  ch.s = amax > 0.0f ? amax / ch.qmaxf : 1.0f;
  ch.rs = 1.0f / ch.s;
  ch.fast = amax >= 0x1p-60f && amax <= 0x1p60f;
  if (tid == 0) d.scales[m] = ch.s;

  // ---- SQuant-C: the composite threshold c_star (candidates at or above it flip) ----
  uint64_t c_star = ~0ull;
  int sgn_c = 0;
  if (kChannelStage) {
    int64_t esum = 0;
    for (size_t n = tid; n < N; n += T) {
      const StreamKernel r = st_solve_kernel<MODE>(ch, n, K);
      esum += r.sum_after;
      count_candidate_bin(sh.hist, r.cand_v);
    }
    const int64_t ec = block_sum(esum, sh.red_i);  // its barriers publish the histogram
    sgn_c = ec > 0 ? 1 : ec < 0 ? -1 : 0;
    int64_t kc = flips_for(ec < 0 ? -ec : ec);
    if (kc > (int64_t)N) kc = (int64_t)N;
    if (kc > 0) {
      // radix select on the composite keys; (composite >> shift) == prefix names the members
      uint32_t need = (uint32_t)kc, need_at = 0, count_at = 0;
      uint32_t digit = scan_histogram_top(sh.hist + (sgn_c < 0 ? 256 : 0), need, need_at, count_at);
      if (digit == kNoDigit) {
        c_star = 1;  // fewer candidates of the wanted sign than flips wanted: all of them flip
      } else {
        uint64_t prefix = digit;
        int shift = 47;  // the top eight of the 23 bits of |v| sit at bits 54..47
        for (;;) {
          need = need_at;
          if (count_at == need || shift == 0) { c_star = prefix << shift; break; }
          if (count_at <= (uint32_t)kStreamListCap) {
            for (size_t n = tid; n < N; n += T) {
              const StreamKernel r = st_solve_kernel<MODE>(ch, n, K);
              const uint64_t comp = st_composite(r.cand_v, sgn_c, n);
              if (comp != 0 && (comp >> shift) == prefix) sh.list[atomicAdd(&sh.list_count, 1u)] = comp;
            }
            __syncthreads();
            if ((uint32_t)tid < count_at) {
              const uint64_t mine = sh.list[tid];
              uint32_t above = 0;
              for (uint32_t e = 0; e < count_at; ++e) above += sh.list[e] > mine ? 1u : 0u;
              if (above == need - 1) sh.result = mine;
            }
            __syncthreads();
            c_star = sh.result;
            break;
          }
          // next digit: bits 46..39, then 38..32 (seven bits), then the index byte by byte
          const int nshift = shift == 47 ? 39 : shift == 39 ? 32 : shift - 8;
          const int width = shift - nshift;
          __syncthreads();  // every wave has finished reading the histogram
          for (int b = tid; b < 256; b += T) sh.hist[b] = 0;
          __syncthreads();
          for (size_t n = tid; n < N; n += T) {
            const StreamKernel r = st_solve_kernel<MODE>(ch, n, K);
            const uint64_t comp = st_composite(r.cand_v, sgn_c, n);
            if (comp != 0 && (comp >> shift) == prefix)
              atomicAdd(&sh.hist[(uint32_t)(comp >> nshift) & ((1u << width) - 1u)], 1u);
          }
          __syncthreads();
          digit = scan_histogram_top(sh.hist, need, need_at, count_at);
          prefix = (prefix << width) | digit;
          shift = nshift;
        }
      }
    }
  }

  // ---- final walk: solve every kernel once more, apply the flips, write the output ----
  // Packed 4-bit output puts two elements in a byte: a thread then takes two consecutive
  // kernels, so that no byte is shared between threads (2K elements start on a byte).
  const int fmt = a.out_format;
  const size_t group = fmt == SQUANT_OUT_INT4 ? 2 : 1;
  const size_t row4 = (L + 1) / 2;
  for (size_t u = tid; u * group < N; u += T) {
    uint32_t pending = 0;
    for (size_t n = u * group; n < u * group + group && n < N; ++n) {
      StreamKernel r;
      r.thr = ~0ull; r.sgn = 0; r.cand_i = -1; r.cand_v = 0; r.sum_after = 0;
      if (MODE != SQUANT_MODE_E) r = st_solve_kernel<MODE>(ch, n, K);
      const uint64_t comp = kChannelStage ? st_composite(r.cand_v, sgn_c, n) : 0;
      const bool cflip = comp != 0 && comp >= c_star;
      const size_t e0 = n * (size_t)K;
      for (int i = 0; i < K; ++i) {
        int code;
        const int32_t P = st_round(ch, e0 + i, code);
        const int32_t aP = r.sgn > 0 ? P : -P;
        if (r.sgn != 0 && aP > 0 && st_key((uint32_t)aP, (uint32_t)i) >= r.thr) code -= r.sgn;
        if (cflip && i == r.cand_i) code -= sgn_c;
        const size_t e = e0 + i;
        if (fmt == SQUANT_OUT_INT8) {
          static_cast<int8_t*>(d.out)[(size_t)m * L + e] = (int8_t)code;
        } else if (fmt == SQUANT_OUT_F32) {
          static_cast<float*>(d.out)[(size_t)m * L + e] = (float)code * ch.s;
        } else if (fmt == SQUANT_OUT_BF16) {
          static_cast<uint16_t*>(d.out)[(size_t)m * L + e] = (uint16_t)bf16_bits((float)code * ch.s);
        } else {
          if ((e & 1) == 0) pending = (uint32_t)code & 0xFu;
          else static_cast<uint8_t*>(d.out)[(size_t)m * row4 + (e >> 1)] = (uint8_t)(pending | (((uint32_t)code & 0xFu) << 4));
          if ((e & 1) == 0 && e + 1 == L)  // an odd row's last element: the high nibble stays 0
            static_cast<uint8_t*>(d.out)[(size_t)m * row4 + (e >> 1)] = (uint8_t)pending;
        }
      }
    }
  }
}

template <int MODE>
__global__ void __launch_bounds__(kStreamThreads) squant_channel_stream(LaunchArgs a) {
  __shared__ StreamShared sh;
  int m;
  const TensorDesc d = locate(a, blockIdx.x, m);
  stream_channel<MODE>(a, d, m, sh);
}

}  // namespace squant
