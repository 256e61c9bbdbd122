// Global-memory access helpers and the output stage shared by the SQuant kernels that keep
// a channel's codes in LDS as biased bytes (code + 128, four to a dword).
#pragma once

#include "squant_common.h"

namespace squant {

typedef float vf3 __attribute__((ext_vector_type(3)));
typedef float vf4 __attribute__((ext_vector_type(4)));
typedef uint32_t vu4 __attribute__((ext_vector_type(4)));
typedef uint32_t vu2 __attribute__((ext_vector_type(2)));

// 16-byte load / store through the global (not flat) address space
__device__ __forceinline__ vf4 load_global_f4(const float* p) {
#if defined(__HIP_DEVICE_COMPILE__)
  return *reinterpret_cast<const __attribute__((address_space(1))) vf4*>(reinterpret_cast<uintptr_t>(p));
#else
  return *reinterpret_cast<const vf4*>(p);
#endif
}
__device__ __forceinline__ vf3 load_global_f3(const float* p) {
#if defined(__HIP_DEVICE_COMPILE__)
  // plain loads: the three 12-byte loads of a kernel share cache lines, and with the
  // non-temporal hint a line is gone by the second touch (measured 6-20 % slower)
  return *reinterpret_cast<const __attribute__((address_space(1))) vf3*>(reinterpret_cast<uintptr_t>(p));
#else
  return *reinterpret_cast<const vf3*>(p);
#endif
}
__device__ __forceinline__ void store_global_u4(void* p, vu4 v) {
#if defined(__HIP_DEVICE_COMPILE__)
  // codes are written once: non-temporal stores (measured 1 % faster)
  __builtin_nontemporal_store(
      v, reinterpret_cast<__attribute__((address_space(1))) vu4*>(reinterpret_cast<uintptr_t>(p)));
#else
  *reinterpret_cast<vu4*>(p) = v;
#endif
}
__device__ __forceinline__ void store_global_u1(void* p, uint32_t v) {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_nontemporal_store(
      v, reinterpret_cast<__attribute__((address_space(1))) uint32_t*>(reinterpret_cast<uintptr_t>(p)));
#else
  *reinterpret_cast<uint32_t*>(p) = v;
#endif
}

__device__ __forceinline__ void store_global_f4(void* p, vf4 v) {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_nontemporal_store(
      v, reinterpret_cast<__attribute__((address_space(1))) vf4*>(reinterpret_cast<uintptr_t>(p)));
#else
  *reinterpret_cast<vf4*>(p) = v;
#endif
}
__device__ __forceinline__ void store_global_u16(void* p, uint16_t v) {
#if defined(__HIP_DEVICE_COMPILE__)
  *reinterpret_cast<__attribute__((address_space(1))) uint16_t*>(reinterpret_cast<uintptr_t>(p)) = v;
#else
  *reinterpret_cast<uint16_t*>(p) = v;
#endif
}

// ---- binary16 / bfloat16 weights: widened exactly to binary32 on load ----
__device__ __forceinline__ float widen_f16(uint32_t bits) {  // low 16 bits
  return (float)__builtin_bit_cast(_Float16, (uint16_t)bits);
}
__device__ __forceinline__ float widen_bf16(uint32_t bits) {  // low 16 bits
  return __uint_as_float(bits << 16);
}
// Both halves of a dword, low half first.
__device__ __forceinline__ void widen_pair(uint32_t d, bool bf16, float& lo, float& hi) {
  if (bf16) {
    lo = __uint_as_float(d << 16);
    hi = __uint_as_float(d & 0xFFFF0000u);
  } else {
    lo = widen_f16(d);
    hi = widen_f16(d >> 16);
  }
}
__device__ __forceinline__ uint32_t load_global_u1(const uint32_t* p) {
#if defined(__HIP_DEVICE_COMPILE__)
  return *reinterpret_cast<const __attribute__((address_space(1))) uint32_t*>(reinterpret_cast<uintptr_t>(p));
#else
  return *p;
#endif
}
__device__ __forceinline__ vu2 load_global_u2_stream(const void* p) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_nontemporal_load(
      reinterpret_cast<const __attribute__((address_space(1))) vu2*>(reinterpret_cast<uintptr_t>(p)));
#else
  return *reinterpret_cast<const vu2*>(p);
#endif
}
// Element i of a weight tensor of the given squant_wtype_t.
__device__ __forceinline__ float load_weight(const void* w, size_t i, int wtype) {
  if (wtype == SQUANT_W_F32) return static_cast<const float*>(w)[i];
  const uint32_t h = static_cast<const uint16_t*>(w)[i];
  return wtype == SQUANT_W_BF16 ? widen_bf16(h) : widen_f16(h);
}

// Low nibbles of the four bytes of c, gathered into 16 bits (byte 0 in bits 0-3).  The
// +128 bias of a code byte does not reach its low nibble, which is the code's 4-bit
// two's complement.
__device__ __forceinline__ uint32_t pack_nibbles4(uint32_t c) {
  uint32_t t = c & 0x0F0F0F0Fu;
  t = (t | (t >> 4)) & 0x00FF00FFu;
  return (t | (t >> 8)) & 0xFFFFu;
}
__device__ __forceinline__ uint32_t pack_nibbles8(uint32_t lo, uint32_t hi) {
  return pack_nibbles4(lo) | (pack_nibbles4(hi) << 16);
}

// The four biased code bytes of c as dequantised weights code * s (Algorithm 1 returns
// C * s; one binary32 multiply per element).
__device__ __forceinline__ vf4 dequant4(uint32_t c, float s) {
  vf4 v;
  v.x = ((float)(c & 0xFFu) - 128.0f) * s;
  v.y = ((float)((c >> 8) & 0xFFu) - 128.0f) * s;
  v.z = ((float)((c >> 16) & 0xFFu) - 128.0f) * s;
  v.w = ((float)(c >> 24) - 128.0f) * s;
  return v;
}

// binary32 to bfloat16 bits, round to nearest, ties to even (finite inputs).
__device__ __forceinline__ uint32_t bf16_bits(float v) {
  const uint32_t b = __float_as_uint(v);
  return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ void store_global_u2(void* p, vu2 v) {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_nontemporal_store(
      v, reinterpret_cast<__attribute__((address_space(1))) vu2*>(reinterpret_cast<uintptr_t>(p)));
#else
  *reinterpret_cast<vu2*>(p) = v;
#endif
}

// Writes output channel m of a tensor from its biased codes in LDS (nvec dwords, so the
// channel has 4 * nvec elements) in the requested format (squant_output_t).  Called by the
// whole workgroup after a barrier; 16-byte stores where the channel's row is aligned.
__device__ __forceinline__ void emit_channel(const uint32_t* code32, int nvec, void* out_base,
                                             int m, float s, int format, int tid, int T) {
  const size_t L = 4 * (size_t)nvec;
  const vu4* src4 = reinterpret_cast<const vu4*>(code32);
  if (format == SQUANT_OUT_INT8) {
    uint8_t* out = static_cast<uint8_t*>(out_base) + (size_t)m * L;
    if ((nvec & 3) == 0 && (reinterpret_cast<uintptr_t>(out) & 15u) == 0) {
      for (int j = tid; j < (nvec >> 2); j += T) store_global_u4(out + 16 * j, src4[j] ^ 0x80808080u);
    } else {
      for (int j = tid; j < nvec; j += T) store_global_u1(out + 4 * j, code32[j] ^ 0x80808080u);
    }
  } else if (format == SQUANT_OUT_INT4) {
    uint8_t* out = static_cast<uint8_t*>(out_base) + (size_t)m * (L / 2);
    if ((nvec & 7) == 0 && (reinterpret_cast<uintptr_t>(out) & 15u) == 0) {
      for (int j = tid; j < (nvec >> 3); j += T) {
        const vu4 a = src4[2 * j], b = src4[2 * j + 1];
        vu4 o;
        o.x = pack_nibbles8(a.x, a.y);
        o.y = pack_nibbles8(a.z, a.w);
        o.z = pack_nibbles8(b.x, b.y);
        o.w = pack_nibbles8(b.z, b.w);
        store_global_u4(out + 16 * j, o);
      }
    } else {
      for (int j = tid; j < nvec; j += T) store_global_u16(out + 2 * j, (uint16_t)pack_nibbles4(code32[j]));
    }
  } else if (format == SQUANT_OUT_BF16) {
    uint16_t* out = static_cast<uint16_t*>(out_base) + (size_t)m * L;
    if ((reinterpret_cast<uintptr_t>(out) & 7u) == 0) {
      for (int j = tid; j < nvec; j += T) {
        const vf4 v = dequant4(code32[j], s);
        vu2 o;
        o.x = bf16_bits(v.x) | (bf16_bits(v.y) << 16);
        o.y = bf16_bits(v.z) | (bf16_bits(v.w) << 16);
        store_global_u2(out + 4 * j, o);
      }
    } else {
      for (int j = tid; j < nvec; j += T) {
        const vf4 v = dequant4(code32[j], s);
        out[4 * j] = (uint16_t)bf16_bits(v.x); out[4 * j + 1] = (uint16_t)bf16_bits(v.y);
        out[4 * j + 2] = (uint16_t)bf16_bits(v.z); out[4 * j + 3] = (uint16_t)bf16_bits(v.w);
      }
    }
  } else {  // SQUANT_OUT_F32
    float* out = static_cast<float*>(out_base) + (size_t)m * L;
    if ((reinterpret_cast<uintptr_t>(out) & 15u) == 0) {
      for (int j = tid; j < nvec; j += T) store_global_f4(out + 4 * j, dequant4(code32[j], s));
    } else {
      for (int j = tid; j < nvec; j += T) {
        const vf4 v = dequant4(code32[j], s);
        out[4 * j] = v.x; out[4 * j + 1] = v.y; out[4 * j + 2] = v.z; out[4 * j + 3] = v.w;
      }
    }
  }
}

// The same output stage for the generic kernel, whose LDS holds plain int8 codes and whose
// channel length L is arbitrary.  A packed row has (L + 1) / 2 bytes; the unused high
// nibble of an odd row's last byte is 0.
__device__ __forceinline__ void emit_channel_bytes(const int8_t* code, int L, void* out_base, int m,
                                                   float s, int format, int tid, int T) {
  if (format == SQUANT_OUT_INT8) {
    int8_t* out = static_cast<int8_t*>(out_base) + (size_t)m * L;
    if ((reinterpret_cast<uintptr_t>(out) & 3u) == 0) {
      const int L4 = L >> 2;
      const uint32_t* src = reinterpret_cast<const uint32_t*>(code);
      uint32_t* dst = reinterpret_cast<uint32_t*>(out);
      for (int j = tid; j < L4; j += T) dst[j] = src[j];
      for (int j = (L4 << 2) + tid; j < L; j += T) out[j] = code[j];
    } else {
      for (int j = tid; j < L; j += T) out[j] = code[j];
    }
  } else if (format == SQUANT_OUT_INT4) {
    const int row = (L + 1) >> 1;
    uint8_t* out = static_cast<uint8_t*>(out_base) + (size_t)m * row;
    for (int j = tid; j < row; j += T) {
      const uint32_t lo = (uint32_t)code[2 * j] & 0xFu;
      const uint32_t hi = (2 * j + 1 < L) ? ((uint32_t)code[2 * j + 1] & 0xFu) : 0u;
      out[j] = (uint8_t)(lo | (hi << 4));
    }
  } else if (format == SQUANT_OUT_BF16) {
    uint16_t* out = static_cast<uint16_t*>(out_base) + (size_t)m * L;
    for (int j = tid; j < L; j += T) out[j] = (uint16_t)bf16_bits((float)code[j] * s);
  } else {  // SQUANT_OUT_F32
    float* out = static_cast<float*>(out_base) + (size_t)m * L;
    for (int j = tid; j < L; j += T) out[j] = (float)code[j] * s;
  }
}

}  // namespace squant
