// Storage formats of (scale, zero) (Section 4.1: FP8 E4M3; Section 4.3 also counts fp16), device
// side.  A pair is stored scale first; element size 4, 2 or 1 byte.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "skvq.h"

namespace skvq {

// float -> FP8 E4M3 (bias 7, largest finite value 448): nearest, ties to even, saturating.
// Done with integer arithmetic so that the result does not depend on a conversion instruction's
// rounding or saturation mode.  Input must not be NaN.
__device__ __forceinline__ unsigned e4m3_from_float(float f) {
  const unsigned sign = (__float_as_uint(f) >> 24) & 0x80u;
  const float a = fabsf(f);
  if (!(a < 448.0f)) return sign | 0x7eu;
  if (a < 0.015625f) return sign | (unsigned)rintf(a * 512.0f);  // subnormals: spacing 2^-9 (8 = first normal)
  unsigned b = __float_as_uint(a);
  b += 0x7ffffu + ((b >> 20) & 1u);  // round the 23-bit mantissa to 3 bits, ties to even
  const unsigned out = (((b >> 23) - 120u) << 3) | ((b >> 20) & 7u);
  return sign | (out > 0x7eu ? 0x7eu : out);
}

// FP8 E4M3 -> float, exact (NaN encodings are never stored).
__device__ __forceinline__ float e4m3_to_float(unsigned b) {
  const unsigned e = (b >> 3) & 15u, m = b & 7u;
  const float v = e ? __uint_as_float(((e + 120u) << 23) | (m << 20)) : (float)m * 0.001953125f;
  return (b & 0x80u) ? -v : v;
}

// A (scale, zero) pair as it reads back from storage, and its storage word (fp16: scale in the
// low half; FP8: scale in the low byte; unused for fp32).
struct MetaPair {
  float scale, zero;
  unsigned stored;
};

__device__ __forceinline__ MetaPair meta_make(float scale, float zero, int fmt) {
  MetaPair m;
  if (fmt == SKVQ_META_F16) {
    const __half2 h = __halves2half2(__float2half_rn(scale), __float2half_rn(zero));
    m.scale = __low2float(h);
    m.zero = __high2float(h);
    m.stored = __builtin_bit_cast(unsigned, h);
  } else if (fmt == SKVQ_META_FP8_E4M3) {
    m.stored = e4m3_from_float(scale) | (e4m3_from_float(zero) << 8);
    m.scale = __builtin_amdgcn_cvt_f32_fp8((int)m.stored, 0);  // decoding is exact
    m.zero = __builtin_amdgcn_cvt_f32_fp8((int)m.stored, 1);
  } else {
    m.scale = scale;
    m.zero = zero;
    m.stored = 0;
  }
  return m;
}

__device__ __forceinline__ void meta_store_pair(void *base, long long pair, const MetaPair &m, int fmt) {
  if (fmt == SKVQ_META_F16)
    reinterpret_cast<unsigned *>(base)[pair] = m.stored;
  else if (fmt == SKVQ_META_FP8_E4M3)
    reinterpret_cast<unsigned short *>(base)[pair] = (unsigned short)m.stored;
  else
    reinterpret_cast<float2 *>(base)[pair] = make_float2(m.scale, m.zero);
}

__device__ __forceinline__ float2 meta_load_pair(const void *base, long long pair, int fmt) {
  if (fmt == SKVQ_META_F16) {
    const __half2 h = reinterpret_cast<const __half2 *>(base)[pair];
    return make_float2(__low2float(h), __high2float(h));
  }
  if (fmt == SKVQ_META_FP8_E4M3) {
    const unsigned w = reinterpret_cast<const unsigned short *>(base)[pair];
    return make_float2(e4m3_to_float(w & 0xffu), e4m3_to_float(w >> 8));
  }
  return reinterpret_cast<const float2 *>(base)[pair];
}

}  // namespace skvq
