// Device-side helpers shared by the gfx950 kernels: vector types, 16-bit conversions, MXFP4 scale
// arithmetic and cross-lane primitives.  CDNA4 only: 64-lane wavefronts, MFMA, LDS.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "thrift.h"

namespace thrift {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef short v4s __attribute__((ext_vector_type(4)));
typedef short v8s __attribute__((ext_vector_type(8)));

constexpr int kD = 128;   // head dimension supported by this version
constexpr int kBk = 64;   // key-block size supported by this version

// ---- 16-bit element traits: the same kernels serve fp16 and bf16 inputs ----
struct F16 {
  typedef _Float16 scalar;
  typedef v8h vec8;
  static __device__ __forceinline__ float to_float(uint16_t u) {
    _Float16 h = __builtin_bit_cast(_Float16, u);
    return (float)h;
  }
  static __device__ __forceinline__ uint16_t from_float(float f) {  // round to nearest even
    _Float16 h = (_Float16)f;
    return __builtin_bit_cast(uint16_t, h);
  }
  // two packed elements -> one byte of E2M1 codes (low nibble = low half), placed in byte `sel` of old
  template <int SEL>
  static __device__ __forceinline__ uint32_t cvt_pk_fp4(uint32_t old, uint32_t pair, float scale) {
    return __builtin_amdgcn_cvt_scalef32_pk_fp4_f16(old, __builtin_bit_cast(v2h, pair), scale, SEL);
  }
  static __device__ __forceinline__ v16f mfma(v8s a, v8s b, v16f c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c, 0, 0, 0);
  }
};

struct BF16 {
  typedef __bf16 scalar;
  typedef v8bf vec8;
  static __device__ __forceinline__ float to_float(uint16_t u) { return __uint_as_float((uint32_t)u << 16); }
  static __device__ __forceinline__ uint16_t from_float(float f) {  // round to nearest even (hardware convert)
    __bf16 h = (__bf16)f;
    return __builtin_bit_cast(uint16_t, h);
  }
  template <int SEL>
  static __device__ __forceinline__ uint32_t cvt_pk_fp4(uint32_t old, uint32_t pair, float scale) {
    return __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(old, __builtin_bit_cast(v2bf, pair), scale, SEL);
  }
  static __device__ __forceinline__ v16f mfma(v8s a, v8s b, v16f c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
  }
};

// ---- E2M1 / E8M0 ----

// Software E2M1 encoder (round to nearest, ties to the even code, saturate at 6, sign kept).  Only
// used where the hardware converter cannot be fed (groups whose scale would be a subnormal float).
__device__ __forceinline__ uint32_t e2m1_encode_sw(float y) {
  uint32_t sign = (__float_as_uint(y) >> 31) << 3;
  float a = fabsf(y);
  uint32_t c = a <= 0.25f ? 0u : a < 0.75f ? 1u : a <= 1.25f ? 2u : a < 1.75f ? 3u : a <= 2.5f ? 4u : a < 3.5f ? 5u : a <= 5.0f ? 6u : 7u;
  return sign | c;
}

// E8M0 byte of a group from the fp32 bit pattern of its largest magnitude (>= 0):
// floor(log2 a) - 2 + 127 for a normal a, clamped below at 0; an all-zero group gets 127.
__device__ __forceinline__ uint32_t e8m0_from_amax_bits(uint32_t amax_bits) {
  if (amax_bits == 0u) return 127u;
  uint32_t ef = amax_bits >> 23;
  return ef >= 2u ? ef - 2u : 0u;
}

// ------------------------------------------------------------------------------------------------
// MXFP4 quantisation of one 32-element group held as 16 packed pairs (pair u = elements 2u, 2u+1).
// Returns the 16 code bytes in out[0..3] and the E8M0 byte.
// ------------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ uint32_t quantize_group32(const uint32_t (&pair)[16], uint32_t (&out)[4]) {
  // magnitudes of 16-bit floats order like their bit patterns without the sign
  uint32_t amax16 = 0;
#pragma unroll
  for (int u = 0; u < 16; ++u) {
    uint32_t lo = pair[u] & 0x7fffu, hi = (pair[u] >> 16) & 0x7fffu;
    amax16 = max(amax16, max(lo, hi));
  }
  const uint32_t abits = __float_as_uint(T::to_float((uint16_t)amax16));
  const uint32_t sb = e8m0_from_amax_bits(abits);
  out[0] = out[1] = out[2] = out[3] = 0u;
  if (sb >= 1u || abits == 0u) {
    // the hardware converter divides by a power-of-two scale given as a normal float
    const float scale = __uint_as_float(sb << 23);
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      uint32_t& o = out[u >> 2];
      switch (u & 3) {
        case 0: o = T::template cvt_pk_fp4<0>(o, pair[u], scale); break;
        case 1: o = T::template cvt_pk_fp4<1>(o, pair[u], scale); break;
        case 2: o = T::template cvt_pk_fp4<2>(o, pair[u], scale); break;
        default: o = T::template cvt_pk_fp4<3>(o, pair[u], scale); break;
      }
    }
  } else {
    // scale 2^-127 is a subnormal float: encode x * 2^127 in software (bf16 groups below 2^-124 only)
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      float lo = T::to_float((uint16_t)(pair[u] & 0xffffu)) * 0x1p64f * 0x1p63f;
      float hi = T::to_float((uint16_t)(pair[u] >> 16)) * 0x1p64f * 0x1p63f;
      out[u >> 2] |= (e2m1_encode_sw(lo) | (e2m1_encode_sw(hi) << 4)) << (8 * (u & 3));
    }
  }
  return sb;
}

// ---- cross-lane ----

// Value held by the lane 32 positions away (lane l <-> lane l^32).
__device__ __forceinline__ float other_half(float x) {
  uint32_t u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  // r[0] = {x.lo, x.lo}, r[1] = {x.hi, x.hi} over (lanes 0-31, lanes 32-63)
  uint32_t lo = r[0], hi = r[1];
  return __uint_as_float((threadIdx.x & 32) ? lo : hi);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

}  // namespace thrift
