// SQuant weight-quantization solver, gfx950 (MI355X) kernels and C ABI.
//
// One workgroup owns one output channel from the first byte read to the last
// byte written: the channel (cin*kh*kw floats) is read from HBM exactly once
// into LDS, the absmax scale, rounding (SQuant-E), kernel-wise flip (SQuant-K),
// candidate update (Algorithm 3) and channel-wise flip (SQuant-C) all run on
// chip, and only int8 codes and one float scale go back to HBM.  Perturbations
// are Q24 integers, so every sum is order independent.
//
// Section / algorithm numbers refer to "SQuant: On-the-Fly Data-Free
// Quantization via Diagonal Hessian Approximation" (ICLR 2022).

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <vector>

#include "squant.h"

namespace {

constexpr int32_t kOne = 1 << 24;   // 1.0 in Q24
constexpr int32_t kHalf = 1 << 23;  // 0.5 in Q24
constexpr int kWave = 64;

struct TensorDesc {
  const float* w;
  int8_t* codes;
  float* scales;
  int32_t M, N, K;
  int32_t first;  // index of this tensor's channel 0 within its launch
};

struct LaunchArgs {
  TensorDesc single;        // used when table == nullptr
  const TensorDesc* table;  // device table, n_tensors entries ordered by `first`
  int32_t n_tensors;
  int32_t uniform_m;        // > 0: every tensor of the table has this many channels
  int32_t qmax;
  int32_t mode;
};

// ---------------------------------------------------------------------------
// small device helpers
// ---------------------------------------------------------------------------

__device__ __forceinline__ TensorDesc locate(const LaunchArgs& a, int g, int& m) {
  if (a.table == nullptr) {
    m = g;
    return a.single;
  }
  int t;
  if (a.uniform_m > 0) {
    t = g / a.uniform_m;
  } else {  // last t with first[t] <= g
    int lo = 0, hi = a.n_tensors - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (a.table[mid].first <= g) lo = mid; else hi = mid - 1;
    }
    t = lo;
  }
  const TensorDesc d = a.table[t];
  m = g - d.first;
  return d;
}

__device__ __forceinline__ int sign_of(int64_t v) { return (v > 0) - (v < 0); }

// k = round(|e|), an exact half rounded down (Algorithm 2, "k = round(|e|)").
__device__ __forceinline__ int64_t flips_for(int64_t abs_sum) { return (abs_sum + kHalf - 1) >> 24; }

// SQuant-E on one scaled weight (Algorithm 1, rounding and element perturbation):
// returns the integer code, writes the Q24 perturbation code - x.
__device__ __forceinline__ int round_and_perturb(float w, float s, float qmaxf, int32_t& P) {
  float x = w / s;  // IEEE binary32 division
  x = fminf(fmaxf(x, -qmaxf), qmaxf);
  const float c = rintf(x);  // round half to even
  const float p = c - x;     // exact
  P = __float2int_rn(p * 16777216.0f);
  return (int)c;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  return v;
}

__device__ __forceinline__ int64_t wave_sum(int64_t v) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

// Every thread returns the block-wide result.  `slot` holds >= 16 entries.
__device__ __forceinline__ float block_max(float v, float* slot) {
  v = wave_max(v);
  const int wid = threadIdx.x / kWave, nw = (blockDim.x + kWave - 1) / kWave;
  __syncthreads();
  if ((threadIdx.x & (kWave - 1)) == 0) slot[wid] = v;
  __syncthreads();
  float r = slot[0];
  for (int i = 1; i < nw; ++i) r = fmaxf(r, slot[i]);
  return r;
}

__device__ __forceinline__ int64_t block_sum(int64_t v, int64_t* slot) {
  v = wave_sum(v);
  const int wid = threadIdx.x / kWave, nw = (blockDim.x + kWave - 1) / kWave;
  __syncthreads();
  if ((threadIdx.x & (kWave - 1)) == 0) slot[wid] = v;
  __syncthreads();
  int64_t r = slot[0];
  for (int i = 1; i < nw; ++i) r += slot[i];
  return r;
}

// Ranking key of a channel-stage candidate: |v| if it has the sign of the channel
// sum, else 0 (not eligible).  0 < key < 2^24 for every eligible candidate.
__device__ __forceinline__ uint32_t cand_key(int32_t v, int sgn) {
  return (sgn > 0 ? v > 0 : v < 0) ? (uint32_t)(v < 0 ? -v : v) : 0u;
}

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
// Generic kernel: any (N, K) whose channel fits in LDS.  One thread per kh*kw
// kernel in the SQuant-K stage, Q24 perturbations and int8 codes held in LDS.
// ---------------------------------------------------------------------------

__global__ void __launch_bounds__(1024) squant_channel_generic(LaunchArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ float red_f[16];
  __shared__ int64_t red_i[16];
  __shared__ uint32_t hist[256];
  __shared__ uint32_t bcast[4];

  int m;
  const TensorDesc d = locate(a, blockIdx.x, m);
  const int N = d.N, K = d.K, L = N * K;
  const int T = blockDim.x, tid = threadIdx.x;
  int32_t* buf = reinterpret_cast<int32_t*>(smem);         // L : weights, then Q24 perturbations
  int32_t* cand = (K == 1) ? buf : buf + L;                // N : candidate perturbation per kernel
  int32_t* cidx = (K == 1) ? nullptr : buf + L + N;        // N : candidate element index
  int8_t* code = reinterpret_cast<int8_t*>(buf + L + (K == 1 ? 0 : 2 * N));  // L codes

  const float* wch = d.w + (size_t)m * L;
  int8_t* out = d.codes + (size_t)m * L;
  const float qmaxf = (float)a.qmax;

  // ---- per-channel absmax (Section 4: per-channel quantization range) ----
  float amax = 0.0f;
  for (int j = tid; j < L; j += T) {
    const float v = wch[j];
    reinterpret_cast<float*>(buf)[j] = v;
    amax = fmaxf(amax, fabsf(v));
  }
  amax = block_max(amax, red_f);
  if (!(amax > 0.0f)) {  // all-zero channel
    for (int j = tid; j < L; j += T) out[j] = 0;
    if (tid == 0) d.scales[m] = 1.0f;
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
    if (K > 1) {
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
        const SelectResult r = radix_select(cand, N, sgn, need, hist, bcast);
        apply_channel_flips(cand, cidx, code, N, K, sgn, r);
      }
    }
  }
  __syncthreads();

  // ---- emit int8 codes ----
  if ((reinterpret_cast<uintptr_t>(out) & 3u) == 0) {
    const int L4 = L >> 2;
    const uint32_t* src = reinterpret_cast<const uint32_t*>(code);
    uint32_t* dst = reinterpret_cast<uint32_t*>(out);
    for (int j = tid; j < L4; j += T) dst[j] = src[j];
    for (int j = (L4 << 2) + tid; j < L; j += T) out[j] = code[j];
  } else {
    for (int j = tid; j < L; j += T) out[j] = code[j];
  }
}

// Copies a chunk of descriptors passed by value into the device table.
constexpr int kDescChunk = 64;
struct DescChunk { TensorDesc t[kDescChunk]; };
__global__ void write_table(DescChunk c, int count, TensorDesc* table) {
  const int i = threadIdx.x;
  if (i < count) table[i] = c.t[i];
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------

struct DeviceLimits { int lds_bytes; bool ok; };

DeviceLimits device_limits() {
  int dev = 0, lds = 0;
  if (hipGetDevice(&dev) != hipSuccess) return {0, false};
  if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess)
    return {0, false};
  return {lds, true};
}

constexpr int kStaticLds = 16 * 4 + 16 * 8 + 256 * 4 + 16 + 64;  // static __shared__ of the kernels, padded

size_t generic_lds_bytes(int64_t N, int64_t K) {
  const int64_t L = N * K;
  return (size_t)(4 * L + (K == 1 ? 0 : 8 * N) + ((L + 3) & ~(int64_t)3) + 16);
}

int generic_threads(int64_t N, int64_t K) {
  const int64_t L = N * K;
  int64_t want = (K == 1) ? (L + 7) / 8 : N;
  want = (want + kWave - 1) / kWave * kWave;
  return (int)std::min<int64_t>(512, std::max<int64_t>(kWave, want));
}

int check_common(int32_t bits, int mode) {
  if (bits < 2 || bits > 8) return SQUANT_ERR_BITS;
  if (mode < SQUANT_MODE_E || mode > SQUANT_MODE_EC) return SQUANT_ERR_MODE;
  return SQUANT_OK;
}

int check_shape(int32_t cout, int32_t cin, int32_t kh, int32_t kw) {
  if (cout <= 0 || cin <= 0 || kh <= 0 || kw <= 0) return SQUANT_ERR_SHAPE;
  const int64_t K = (int64_t)kh * kw;
  const int64_t L = K * cin;
  if (K > (1 << 20) || L > (int64_t)1 << 30) return SQUANT_ERR_SHAPE;
  return SQUANT_OK;
}

struct Group {
  int threads;
  size_t lds;
  std::vector<TensorDesc> t;
};

int launch_group(const Group& g, const TensorDesc* d_table, int qmax, int mode, hipStream_t st) {
  LaunchArgs a{};
  int64_t total = 0;
  bool uniform = true;
  for (const auto& t : g.t) { total += t.M; uniform &= (t.M == g.t[0].M); }
  if (total <= 0 || total > 0x7fffffff) return SQUANT_ERR_SHAPE;
  if (d_table == nullptr) {
    a.single = g.t[0];
    a.table = nullptr;
    a.n_tensors = 1;
  } else {
    a.table = d_table;
    a.n_tensors = (int)g.t.size();
  }
  a.uniform_m = uniform ? g.t[0].M : 0;
  a.qmax = qmax;
  a.mode = mode;
  if (g.lds > 48 * 1024) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(squant_channel_generic),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)g.lds) != hipSuccess) {
      (void)hipGetLastError();
      return SQUANT_ERR_DEVICE;
    }
  }
  hipLaunchKernelGGL(squant_channel_generic, dim3((unsigned)total), dim3(g.threads), g.lds, st, a);
  if (hipGetLastError() != hipSuccess) return SQUANT_ERR_DEVICE;
  return SQUANT_OK;
}

}  // namespace

extern "C" {

int squant_quantize(const float* d_w, int32_t cout, int32_t cin, int32_t kh, int32_t kw,
                    int32_t bits, squant_mode_t mode, int8_t* d_codes, float* d_scales,
                    void* stream) {
  if (!d_w || !d_codes || !d_scales) return SQUANT_ERR_NULL;
  if (int rc = check_shape(cout, cin, kh, kw)) return rc;
  if (int rc = check_common(bits, (int)mode)) return rc;
  const DeviceLimits lim = device_limits();
  if (!lim.ok) { (void)hipGetLastError(); return SQUANT_ERR_DEVICE; }
  const int64_t K = (int64_t)kh * kw;
  Group g;
  g.lds = generic_lds_bytes(cin, K);
  if (g.lds + kStaticLds > (size_t)lim.lds_bytes) return SQUANT_ERR_UNSUPPORTED;
  g.threads = generic_threads(cin, K);
  g.t.push_back(TensorDesc{d_w, d_codes, d_scales, cout, cin, (int32_t)K, 0});
  return launch_group(g, nullptr, (1 << (bits - 1)) - 1, (int)mode, (hipStream_t)stream);
}

size_t squant_batched_workspace_bytes(int32_t n_tensors) {
  if (n_tensors <= 0) return 0;
  return (size_t)n_tensors * sizeof(TensorDesc);
}

int squant_quantize_batched(const squant_tensor_t* h_tensors, int32_t n_tensors, int32_t bits,
                            squant_mode_t mode, void* d_workspace, size_t workspace_bytes,
                            void* stream) {
  if (n_tensors < 0) return SQUANT_ERR_SHAPE;
  if (n_tensors == 0) return SQUANT_OK;
  if (!h_tensors) return SQUANT_ERR_NULL;
  if (int rc = check_common(bits, (int)mode)) return rc;
  for (int32_t i = 0; i < n_tensors; ++i) {
    const squant_tensor_t& t = h_tensors[i];
    if (!t.w || !t.codes || !t.scales) return SQUANT_ERR_NULL;
    if (int rc = check_shape(t.cout, t.cin, t.kh, t.kw)) return rc;
  }
  if (!d_workspace || workspace_bytes < squant_batched_workspace_bytes(n_tensors) ||
      (reinterpret_cast<uintptr_t>(d_workspace) & 15u) != 0)
    return SQUANT_ERR_WORKSPACE;
  const DeviceLimits lim = device_limits();
  if (!lim.ok) { (void)hipGetLastError(); return SQUANT_ERR_DEVICE; }

  // group tensors by launch configuration
  std::vector<Group> groups;
  for (int32_t i = 0; i < n_tensors; ++i) {
    const squant_tensor_t& t = h_tensors[i];
    const int64_t K = (int64_t)t.kh * t.kw;
    const size_t lds = generic_lds_bytes(t.cin, K);
    if (lds + kStaticLds > (size_t)lim.lds_bytes) return SQUANT_ERR_UNSUPPORTED;
    const int threads = generic_threads(t.cin, K);
    // LDS size classes: next power of two >= 2 KB keeps the number of launches small
    size_t cls = 2048;
    while (cls < lds) cls <<= 1;
    cls = std::min(cls, (size_t)lim.lds_bytes - kStaticLds);
    Group* g = nullptr;
    for (auto& c : groups) if (c.threads == threads && c.lds == cls) { g = &c; break; }
    if (!g) { groups.push_back(Group{threads, cls, {}}); g = &groups.back(); }
    int64_t first = 0;
    if (!g->t.empty()) first = (int64_t)g->t.back().first + g->t.back().M;
    if (first + t.cout > 0x7fffffff) return SQUANT_ERR_SHAPE;
    g->t.push_back(TensorDesc{t.w, t.codes, t.scales, t.cout, t.cin, (int32_t)K, (int32_t)first});
  }

  hipStream_t st = (hipStream_t)stream;
  TensorDesc* table = static_cast<TensorDesc*>(d_workspace);
  size_t offset = 0;
  const int qmax = (1 << (bits - 1)) - 1;
  for (const auto& g : groups) {
    for (size_t c0 = 0; c0 < g.t.size(); c0 += kDescChunk) {
      DescChunk chunk{};
      const int cnt = (int)std::min<size_t>(kDescChunk, g.t.size() - c0);
      for (int i = 0; i < cnt; ++i) chunk.t[i] = g.t[c0 + i];
      hipLaunchKernelGGL(write_table, dim3(1), dim3(kDescChunk), 0, st, chunk, cnt,
                         table + offset + c0);
      if (hipGetLastError() != hipSuccess) return SQUANT_ERR_DEVICE;
    }
    if (int rc = launch_group(g, table + offset, qmax, (int)mode, st)) return rc;
    offset += g.t.size();
  }
  return SQUANT_OK;
}

int64_t squant_max_channel_elems(int32_t kh, int32_t kw) {
  if (kh <= 0 || kw <= 0) return 0;
  const DeviceLimits lim = device_limits();
  if (!lim.ok) { (void)hipGetLastError(); return 0; }
  const int64_t K = (int64_t)kh * kw;
  // largest N with generic_lds_bytes(N, K) + static <= limit
  const int64_t budget = (int64_t)lim.lds_bytes - kStaticLds - 16 - 3;
  const int64_t per_kernel = 5 * K + (K == 1 ? 0 : 8);
  const int64_t n = budget / per_kernel;
  return n > 0 ? n * K : 0;
}

const char* squant_status_string(int status) {
  switch (status) {
    case SQUANT_OK: return "ok";
    case SQUANT_ERR_NULL: return "null pointer";
    case SQUANT_ERR_SHAPE: return "bad shape";
    case SQUANT_ERR_BITS: return "bits must be in [2, 8]";
    case SQUANT_ERR_MODE: return "unknown mode";
    case SQUANT_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case SQUANT_ERR_DEVICE: return "HIP call failed";
    case SQUANT_ERR_UNSUPPORTED: return "output channel too large for one workgroup's LDS";
    default: return "unknown status";
  }
}

int squant_version(void) { return 100; }

}  // extern "C"
