// Device code of the two-pass MXFP4 block decomposition (paper Sec. 3.2.1, Alg. 2), shared by
// the stand-alone decomposition kernel and by the single-launch W4A16 decode GEMM.
#pragma once
#include "msd_common.hpp"

namespace msd {

// Exponent e of alpha = 2^e for a block with max-abs mb: smallest e with mb <= hi * 2^(e + ebias), read
// off the fp32 fields (hi in [1, 2) given by its mantissa field: 1.859375 is 0x6E0000, 1.75 is
// 0x600000, 1.5 is 0x400000); clamped to [-123, 127].
__device__ __forceinline__ int mx_alpha_exponent(float mb, const MxVariant& mv) {
  const uint32_t u = __float_as_uint(mb);
  int e = (int)(u >> 23) - 127 - mv.ebias;
  if ((u & 0x7FFFFFu) > mv.hi_mant) e += 1;
  return min(max(e, -123), 127);
}

__device__ __forceinline__ float pow2f(int e) {  // e in [-126, 127]
  return __uint_as_float((uint32_t)(e + 127) << 23);
}

__device__ __forceinline__ float block_absmax(const uint32_t (&w)[16]) {
  float mb = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    mb = fmaxf(mb, fabsf(__uint_as_float(w[i] << 16)));
    mb = fmaxf(mb, fabsf(__uint_as_float(w[i] & 0xFFFF0000u)));
  }
  return mb;
}

// Nearest value of the MX FP4 element grid to v (exact input), ties to the even code, saturating at
// 6: rounding to nearest-even on the local spacing (0.5 below 2, 1 below 4, 2 above) is exactly
// that.  Returns the value; code = its signed magnitude code (0..7: 0, .5, 1, 1.5, 2, 3, 4, 6).
__device__ __forceinline__ float e2m1_round(float v, int& code) {
  const float a = fabsf(v);
  const float inv_g = a < 2.f ? 2.f : (a < 4.f ? 1.f : 0.5f);
  const float g = a < 2.f ? 0.5f : (a < 4.f ? 1.f : 2.f);
  const float q = fminf(rintf(a * inv_g) * g, 6.f);
  const int h = (int)(q * 2.f);                 // value in halves: 0, 1, 2, 3, 4, 6, 8, 12
  const int c = h <= 4 ? h : (h >> 2) + 4;
  code = v < 0.f ? -c : c;
  return v < 0.f ? -q : q;
}

// One element: both passes.  Returns the two signed codes: on the uniform grid the integers k1, k2
// (value k/4, |k| <= 7); on the E2M1 grid the signed magnitude codes (|c| <= 7).
__device__ __forceinline__ void mx_element_codes(float x, int e, const MxVariant& mv, int& c1, int& c2) {
  if (mv.e2m1) {
    const float inv_alpha = pow2f(-e), alpha = pow2f(e);  // e <= 126 whenever the block is finite
    const float q = e2m1_round(x * inv_alpha, c1);
    const float r = __fmaf_rn(-q, alpha, x);  // exact
    (void)e2m1_round(r * inv_alpha * pow2f(mv.shift), c2);
  } else {
    const float up = pow2f(2 - e);    // 4/alpha
    const float down = pow2f(e - 2);  // alpha/4
    const float a = fminf(fmaxf(rintf(x * up), -7.f), 7.f);
    const float r = __fmaf_rn(-a, down, x);  // exact
    const float b = fminf(fmaxf(rintf(r * up * pow2f(mv.shift)), -7.f), 7.f);
    c1 = (int)a;
    c2 = (int)b;
  }
}

// 32 BF16 values of one block -> signed codes of both components and the exponent e of alpha
// (beta = alpha / 2^shift).
__device__ __forceinline__ int mx_block_codes(const uint32_t (&w)[16], int (&k1)[32], int (&k2)[32],
                                              const MxVariant& mv) {
  const int e = mx_alpha_exponent(block_absmax(w), mv);
#pragma unroll
  for (int i = 0; i < 32; ++i) {
    const float x = (i & 1) ? __uint_as_float(w[i >> 1] & 0xFFFF0000u) : __uint_as_float(w[i >> 1] << 16);
    mx_element_codes(x, e, mv, k1[i], k2[i]);
  }
  return e;
}

// Signed code -> the 6-bit FP6 E2M3 operand code of its value.  Uniform grid: value k/4 has
// magnitude field 2|k|.  E2M1 grid: the E2M1 magnitude code (exponent, mantissa bit) keeps its
// exponent and puts the mantissa bit on top of the three: field = code << 2.
__device__ __forceinline__ uint32_t e2m3_code(int k, int e2m1) {
  const uint32_t mag = (uint32_t)(k < 0 ? -k : k);
  return (k < 0 ? 32u : 0u) | (e2m1 ? mag << 2 : mag << 1);
}

// Same decomposition, packed on the fly: 32 BF16 values -> the FP6-E2M3 operands of both
// components (6 dwords each, element i at bits [6i, 6i+6)) and the exponent e.  Keeps no
// 32-element code arrays alive (the GEMM kernels that decompose in place are register-bound).
__device__ __forceinline__ int mx_block_pack_fp6(const uint32_t (&w)[16], uint32_t (&p1)[6], uint32_t (&p2)[6],
                                                 const MxVariant& mv) {
  const int e = mx_alpha_exponent(block_absmax(w), mv);
#pragma unroll
  for (int h = 0; h < 2; ++h) {  // 16 codes -> 96 bits -> 3 dwords per component
    uint64_t lo1 = 0, lo2 = 0;
    uint32_t hi1 = 0, hi2 = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int idx = h * 16 + i;
      const float x = (idx & 1) ? __uint_as_float(w[idx >> 1] & 0xFFFF0000u) : __uint_as_float(w[idx >> 1] << 16);
      int ka, kb;
      mx_element_codes(x, e, mv, ka, kb);
      const uint64_t c1 = e2m3_code(ka, mv.e2m1);
      const uint64_t c2 = e2m3_code(kb, mv.e2m1);
      const int bit = 6 * i;
      if (bit + 6 <= 64) {
        lo1 |= c1 << bit;
        lo2 |= c2 << bit;
      } else if (bit >= 64) {
        hi1 |= (uint32_t)c1 << (bit - 64);
        hi2 |= (uint32_t)c2 << (bit - 64);
      } else {  // straddles bit 64 (i = 10: bits 60..65)
        lo1 |= c1 << bit;
        lo2 |= c2 << bit;
        hi1 |= (uint32_t)(c1 >> (64 - bit));
        hi2 |= (uint32_t)(c2 >> (64 - bit));
      }
    }
    p1[h * 3 + 0] = (uint32_t)lo1; p1[h * 3 + 1] = (uint32_t)(lo1 >> 32); p1[h * 3 + 2] = hi1;
    p2[h * 3 + 0] = (uint32_t)lo2; p2[h * 3 + 1] = (uint32_t)(lo2 >> 32); p2[h * 3 + 2] = hi2;
  }
  return e;
}

// ABI nibble of a signed code (either grid): bit 3 sign, bits 2..0 magnitude code, -0 -> +0
__device__ __forceinline__ uint32_t nibble4(int k) {
  return k < 0 ? (8u | (uint32_t)(-k)) : (uint32_t)k;
}

// Pack 32 six-bit codes into 6 dwords, element i at bits [6i, 6i+6).
__device__ __forceinline__ void pack_fp6(const int (&k)[32], uint32_t (&out)[6], int e2m1) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {  // 16 codes -> 96 bits -> 3 dwords
    uint64_t lo = 0;             // bits 0..63
    uint32_t hi = 0;             // bits 64..95
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const uint64_t c = e2m3_code(k[h * 16 + i], e2m1);
      const int bit = 6 * i;
      if (bit + 6 <= 64) {
        lo |= c << bit;
      } else if (bit >= 64) {
        hi |= (uint32_t)c << (bit - 64);
      } else {  // straddles bit 64 (i = 10: bits 60..65)
        lo |= c << bit;
        hi |= (uint32_t)(c >> (64 - bit));
      }
    }
    out[h * 3 + 0] = (uint32_t)lo;
    out[h * 3 + 1] = (uint32_t)(lo >> 32);
    out[h * 3 + 2] = hi;
  }
}

}  // namespace msd
