// Generic SQuant kernel: any (cin, kh*kw) whose output channel fits in LDS.
#pragma once

#include "squant_common.h"
#include "squant_io.h"
#include "squant_select.h"

namespace squant {

// Block-level radix select over the N per-kernel candidates of one channel
// (SQuant-C, Algorithm 2 applied to the channel): finds the key value T of the
// `need`-th largest eligible candidate, three 8-bit digits from the top, with a
// 256-bin LDS histogram per digit.  On return every key > T is to be flipped,
// and `need_at_t` of the `count_at_t` keys equal to T (lowest kernel index first).
// If fewer than `need` candidates are eligible, T = 1 and all of them flip.
struct SelectResult { uint32_t T; uint32_t need_at_t; uint32_t count_at_t; };

__device__ SelectResult radix_select(const int32_t* cand, int N, int sgn, uint32_t need,
                                     uint32_t* hist, uint32_t* bcast) {
  uint32_t prefix = 0;
  uint32_t count_at = 0;
  for (int pass = 0; pass < 3; ++pass) {
    const int shift = 16 - 8 * pass;
    for (int b = threadIdx.x; b < 256; b += blockDim.x) hist[b] = 0;
    __syncthreads();
    for (int n = threadIdx.x; n < N; n += blockDim.x) {
      const uint32_t key = cand_key(cand[n], sgn);
      if (key != 0 && (pass == 0 || (key >> (shift + 8)) == prefix))
        atomicAdd(&hist[(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (threadIdx.x < kWave) {
      // lane l owns bins 4l..4l+3; suffix sums over lanes find the digit at which the
      // count of keys with a larger-or-equal digit first reaches `need`
      const int l = threadIdx.x;
      const uint32_t h0 = hist[4 * l], h1 = hist[4 * l + 1], h2 = hist[4 * l + 2], h3 = hist[4 * l + 3];
      const uint32_t mine = h0 + h1 + h2 + h3;
      uint32_t suf = mine;  // inclusive suffix sum: lanes >= l
#pragma unroll
      for (int off = 1; off < kWave; off <<= 1) {
        const uint32_t o = __shfl_down(suf, off);
        if (l + off < kWave) suf += o;
      }
      const unsigned long long reach = __ballot(suf >= need);
      if (reach == 0ull) {  // fewer eligible candidates than flips wanted: take them all
        if (l == 0) { bcast[0] = 0xFFFFFFFFu; bcast[1] = 0; bcast[2] = 0; }
      } else {
        const int top = 63 - __builtin_clzll(reach);
        if (l == top) {
          uint32_t above = suf - mine;  // keys in higher lanes' bins
          uint32_t digit, cnt;
          if (above + h3 >= need) { digit = 4 * l + 3; cnt = h3; }
          else if (above + h3 + h2 >= need) { digit = 4 * l + 2; cnt = h2; above += h3; }
          else if (above + h3 + h2 + h1 >= need) { digit = 4 * l + 1; cnt = h1; above += h3 + h2; }
          else { digit = 4 * l; cnt = h0; above += h3 + h2 + h1; }
          bcast[0] = digit; bcast[1] = need - above; bcast[2] = cnt;
        }
      }
    }
    __syncthreads();
    const uint32_t digit = bcast[0];
    if (digit == 0xFFFFFFFFu) return SelectResult{1u, 0u, 0u};  // only reachable in pass 0
    need = bcast[1];
    count_at = bcast[2];
    prefix = (prefix << 8) | digit;
    __syncthreads();
  }
  return SelectResult{prefix, need, count_at};
}

// Applies the channel-wise flips chosen by radix_select to the int8 codes in LDS.
// `cidx` = per-kernel candidate element index (nullptr when K == 1).
__device__ void apply_channel_flips(const int32_t* cand, const int32_t* cidx, int8_t* code, int N,
                                    int K, int sgn, SelectResult r) {
  const bool all_ties = (r.need_at_t == r.count_at_t);
  for (int n = threadIdx.x; n < N; n += blockDim.x) {
    const uint32_t key = cand_key(cand[n], sgn);
    if (key != 0 && (key > r.T || (all_ties && key == r.T))) {
      const int j = n * K + (cidx ? cidx[n] : 0);
      code[j] = (int8_t)(code[j] - sgn);
    }
  }
  if (!all_ties && threadIdx.x < kWave) {
    // some, not all, of the keys equal to T flip: lowest kernel index first
    uint32_t left = r.need_at_t;
    const int l = threadIdx.x;
    for (int base = 0; base < N && left > 0; base += kWave) {
      const int n = base + l;
      const bool eq = n < N && cand_key(cand[n], sgn) == r.T;
      const unsigned long long mask = __ballot(eq);
      const uint32_t rank = (uint32_t)__popcll(mask & ((1ull << l) - 1ull));
      if (eq && rank < left) {
        const int j = n * K + (cidx ? cidx[n] : 0);
        code[j] = (int8_t)(code[j] - sgn);
      }
      const uint32_t got = (uint32_t)__popcll(mask);
      left = got >= left ? 0u : left - got;
    }
  }
}

// ---------------------------------------------------------------------------
// SQuant-K and the candidate update for ONE kernel by ONE wave (large kh*kw, e.g. a
// 7x7 stem): element i sits with lane i % 64.  The k-th largest same-sign |p| is
// found by a wavefront-level radix select, one ballot + population count per key bit
// from the top (Algorithm 2's top-k); elements above it flip, and of those equal to it
// the lowest indices (ballot prefix ranks).  Everything the wave decides is uniform.
//   pk, ck   the kernel's K perturbations (Q23) and codes in LDS, updated in place
//   returns  the kernel's perturbation sum after the flips; cv / ci = Algorithm 3 candidate
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint32_t same_sign_key(int32_t p, int sgn) {
  const int32_t a = sgn > 0 ? p : -p;
  return a > 0 ? (uint32_t)a : 0u;  // 0 = not eligible
}

__device__ int64_t kernel_stage_wave(int32_t* pk, int8_t* ck, int K, int mode, int32_t& cv,
                                     int32_t& ci) {
  const int lane = threadIdx.x & (kWave - 1);
  const unsigned long long below = (1ull << lane) - 1ull;
  int64_t part = 0;
  for (int i = lane; i < K; i += kWave) part += pk[i];
  int64_t e = wave_sum(part);
  const int sgn = sign_of(e);
  const int64_t A = e < 0 ? -e : e;
  const uint32_t k = (mode == SQUANT_MODE_EC) ? 0u : (uint32_t)flips_for(A);
  cv = 0;
  ci = 0;
  if (sgn == 0) {  // nothing masked: largest |p| of either sign, lowest index
    uint32_t best = 0;
    for (int i = lane; i < K; i += kWave) {
      const int32_t p = pk[i];
      best = max(best, (uint32_t)(p < 0 ? -p : p));
    }
    best = (uint32_t)__builtin_amdgcn_readlane((int)wave_prefix_max_u32(best), kWave - 1);
    if (best != 0) {
      for (int base = 0; base < K; base += kWave) {
        const int i = base + lane;
        const int32_t p = i < K ? pk[i] : 0;
        const unsigned long long hit = __ballot(i < K && (uint32_t)(p < 0 ? -p : p) == best);
        if (hit) {
          const int l = __builtin_ctzll(hit);
          ci = base + l;
          cv = __builtin_amdgcn_readlane(p, l);
          break;
        }
      }
    }
    return e;
  }

  uint32_t T = 0xFFFFFFFFu;  // key of the k-th largest same-sign element (nothing flips if k = 0)
  uint32_t take_eq = 0;      // how many of the elements with key == T flip
  if (k > 0) {
    // kernels of up to 256 elements keep their keys in registers for the 23 steps (a 7x7
    // kernel: one register per lane) instead of reading LDS in every step
    constexpr int kRegChunks = 4;
    const bool in_regs = K <= kRegChunks * kWave;
    uint32_t kreg[kRegChunks];
#pragma unroll
    for (int r = 0; r < kRegChunks; ++r) {
      const int i = r * kWave + lane;
      kreg[r] = (in_regs && i < K) ? same_sign_key(pk[i], sgn) : 0u;
    }
    uint32_t prefix = 0, need = k;
    for (int b = 22; b >= 0; --b) {
      const uint32_t want = (prefix << 1) | 1u;
      uint32_t cnt = 0;
      if (in_regs) {
#pragma unroll
        for (int r = 0; r < kRegChunks; ++r)
          if (r * kWave < K) cnt += (uint32_t)__popcll(__ballot(kreg[r] != 0 && (kreg[r] >> b) == want));
      } else {
        for (int base = 0; base < K; base += kWave) {
          const int i = base + lane;
          const uint32_t key = i < K ? same_sign_key(pk[i], sgn) : 0u;
          cnt += (uint32_t)__popcll(__ballot(key != 0 && (key >> b) == want));
        }
      }
      if (cnt >= need) prefix = want; else { need -= cnt; prefix <<= 1; }
    }
    T = prefix;
    take_eq = need;
  }

  // flip pass; remembers the last flipped element (over SQuant) and the first un-flipped
  // element equal to T, if any (under SQuant)
  uint32_t eq_before = 0;
  int over_i = -1, under_i = -1;
  for (int base = 0; base < K && k > 0; base += kWave) {
    const int i = base + lane;
    const int32_t p = i < K ? pk[i] : 0;
    const uint32_t key = i < K ? same_sign_key(p, sgn) : 0u;
    const bool eq = key != 0 && key == T;
    const unsigned long long eqmask = __ballot(eq);
    const uint32_t rank = eq_before + (uint32_t)__popcll(eqmask & below);
    const bool take = key != 0 && (key > T || (eq && rank < take_eq));
    if (take) {
      pk[i] = p - sgn * kOne;
      ck[i] = (int8_t)(ck[i] - sgn);
    }
    const unsigned long long last = __ballot(eq && rank == take_eq - 1);
    if (last) over_i = base + __builtin_ctzll(last);
    const unsigned long long next = __ballot(eq && rank == take_eq);
    if (next && under_i < 0) under_i = base + __builtin_ctzll(next);
    eq_before += (uint32_t)__popcll(eqmask);
  }
  e -= (int64_t)sgn * (int64_t)k * kOne;

  if ((int64_t)k * kOne > A) {  // over SQuant: the last flipped element, post-flip value
    if (over_i >= 0) { ci = over_i; cv = pk[over_i]; }
    return e;
  }
  // under SQuant: the first un-flipped same-sign element
  if (under_i >= 0) { ci = under_i; cv = pk[under_i]; return e; }
  uint32_t best = 0;  // largest same-sign key below T (all keys >= T have flipped sign by now)
  for (int i = lane; i < K; i += kWave) {
    const uint32_t key = same_sign_key(pk[i], sgn);
    if (key < T) best = max(best, key);
  }
  best = (uint32_t)__builtin_amdgcn_readlane((int)wave_prefix_max_u32(best), kWave - 1);
  if (best != 0) {
    for (int base = 0; base < K; base += kWave) {
      const int i = base + lane;
      const int32_t p = i < K ? pk[i] : 0;
      const unsigned long long hit = __ballot(i < K && same_sign_key(p, sgn) == best);
      if (hit) {
        const int l = __builtin_ctzll(hit);
        ci = base + l;
        cv = __builtin_amdgcn_readlane(p, l);
        break;
      }
    }
  }
  return e;
}

// ---------------------------------------------------------------------------
// Generic kernel: any (N, K) whose channel fits in LDS.  Q23 perturbations and int8
// codes are held in LDS; the SQuant-K stage takes one thread per kh*kw kernel for small
// kernels and one wave per kernel from kWaveKernelMinK elements on.
// ---------------------------------------------------------------------------
constexpr int kWaveKernelMinK = 32;

struct GenericShared {
  float red_f[16];
  int64_t red_i[16];
  uint32_t hist[256];
  uint32_t bcast[4];
};

__device__ __forceinline__ void generic_channel(const LaunchArgs& a, const TensorDesc& d, int m,
                                                unsigned char* smem, GenericShared& gs) {
  float* red_f = gs.red_f;
  int64_t* red_i = gs.red_i;
  uint32_t* hist = gs.hist;
  uint32_t* bcast = gs.bcast;
  const int N = d.N, K = d.K, L = N * K;
  const int T = blockDim.x, tid = threadIdx.x;
  int32_t* buf = reinterpret_cast<int32_t*>(smem);         // L : weights, then Q23 perturbations
  int32_t* cand = (K == 1) ? buf : buf + L;                // N : candidate perturbation per kernel
  int32_t* cidx = (K == 1) ? nullptr : buf + L + N;        // N : candidate element index
  int8_t* code = reinterpret_cast<int8_t*>(buf + L + (K == 1 ? 0 : 2 * N));  // L codes

  const float qmaxf = (float)a.qmax;

  // ---- per-channel absmax (Section 4: per-channel quantization range) ----
  float amax = 0.0f;
  for (int j = tid; j < L; j += T) {
    const float v = load_weight(d.w, (size_t)m * L + j, a.wtype);
    reinterpret_cast<float*>(buf)[j] = v;
    amax = fmaxf(amax, fabsf(v));
  }
  amax = block_max(amax, red_f);
  if (!(amax > 0.0f)) {  // all-zero channel
    for (int j = tid; j < L; j += T) code[j] = 0;
    if (tid == 0) d.scales[m] = 1.0f;
    __syncthreads();
    emit_channel_bytes(code, L, d.out, m, 1.0f, a.out_format, tid, T);
    return;
  }
  const float s = amax / qmaxf;
  if (tid == 0) d.scales[m] = s;

  // ---- SQuant-E ----
  int64_t esum = 0;
  for (int j = tid; j < L; j += T) {
    int32_t P;
    const int c = round_and_perturb(reinterpret_cast<float*>(buf)[j], s, qmaxf, P);
    buf[j] = P;
    code[j] = (int8_t)c;
    esum += P;
  }
  __syncthreads();

  if (a.mode != SQUANT_MODE_E) {
    if (K >= kWaveKernelMinK) {
      // ---- SQuant-K and the candidate update, one wave per kernel ----
      esum = 0;
      const int wid = tid / kWave, nw = T / kWave;
      for (int n = wid; n < N; n += nw) {
        int32_t cv, ci;
        const int64_t e = kernel_stage_wave(buf + n * K, code + n * K, K, a.mode, cv, ci);
        if ((tid & (kWave - 1)) == 0) {
          esum += e;
          cand[n] = cv;
          cidx[n] = ci;
        }
      }
    } else if (K > 1) {
      // ---- SQuant-K and the candidate update, one thread per kernel ----
      esum = 0;
      for (int n = tid; n < N; n += T) {
        int32_t* pk = buf + n * K;
        int8_t* ck = code + n * K;
        int64_t e = 0;
        for (int i = 0; i < K; ++i) e += pk[i];
        const int sgn = sign_of(e);
        const int64_t A = e < 0 ? -e : e;
        const int64_t k = (a.mode == SQUANT_MODE_EC) ? 0 : flips_for(A);
        int last = -1;
        for (int64_t r = 0; r < k; ++r) {
          // largest same-sign |p| not yet flipped (a flipped element changes sign)
          int best = -1, best_abs = 0;
          for (int i = 0; i < K; ++i) {
            const int32_t p = pk[i];
            const int ap = sgn > 0 ? p : -p;  // > 0 iff same sign
            if (ap > best_abs) { best_abs = ap; best = i; }
          }
          if (best < 0) break;  // cannot happen for finite input (App. B.1)
          pk[best] -= sgn * kOne;
          ck[best] = (int8_t)(ck[best] - sgn);
          e -= (int64_t)sgn * kOne;
          last = best;
        }
        esum += e;
        int ci = 0;
        int32_t cv = 0;
        if (sgn == 0) {  // nothing masked: largest |p| of either sign
          int best_abs = 0;
          for (int i = 0; i < K; ++i) {
            const int32_t p = pk[i];
            const int ap = p < 0 ? -p : p;
            if (ap > best_abs) { best_abs = ap; ci = i; cv = p; }
          }
        } else if (k * kOne > A) {  // over SQuant: last flipped element, post-flip value
          if (last >= 0) { ci = last; cv = pk[last]; }
        } else {  // under SQuant: first un-flipped same-sign element
          int best_abs = 0;
          for (int i = 0; i < K; ++i) {
            const int32_t p = pk[i];
            const int ap = sgn > 0 ? p : -p;
            if (ap > best_abs) { best_abs = ap; ci = i; cv = p; }
          }
        }
        cand[n] = cv;
        cidx[n] = ci;
      }
    }
    if (a.mode == SQUANT_MODE_EKC || a.mode == SQUANT_MODE_EC) {
      // ---- SQuant-C ----
      const int64_t ec = block_sum(esum, red_i);  // barriers inside also publish cand/cidx
      const int sgn = sign_of(ec);
      const int64_t kc = flips_for(ec < 0 ? -ec : ec);
      if (kc > 0) {
        const uint32_t need = (uint32_t)(kc > (int64_t)N ? (int64_t)N : kc);
        if (N <= kWave) {
          // few kernels (a 7x7 stem has three): lane n of the first wave holds candidate n and
          // ranks it against the others directly, larger |v| first, then lower kernel index
          if (tid < kWave) {
            const uint32_t key = tid < N ? cand_key(cand[tid], sgn) : 0u;
            uint32_t rank = 0;
            for (int o = 0; o < N; ++o) {
              const uint32_t ko = (uint32_t)__builtin_amdgcn_readlane((int)key, o);
              rank += (ko > key || (ko == key && o < tid)) ? 1u : 0u;
            }
            if (key != 0 && rank < need) {
              const int j = tid * K + (cidx ? cidx[tid] : 0);
              code[j] = (int8_t)(code[j] - sgn);
            }
          }
        } else {
          const SelectResult r = radix_select(cand, N, sgn, need, hist, bcast);
          apply_channel_flips(cand, cidx, code, N, K, sgn, r);
        }
      }
    }
  }
  __syncthreads();

  emit_channel_bytes(code, L, d.out, m, s, a.out_format, tid, T);
}

__global__ void __launch_bounds__(1024) squant_channel_generic(LaunchArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ GenericShared gs;
  int m;
  const TensorDesc d = locate(a, blockIdx.x, m);
  generic_channel(a, d, m, smem, gs);
}

}  // namespace squant
