// Device code of the two-pass MXFP4 block decomposition (paper Sec. 3.2.1, Alg. 2), shared by
// the stand-alone decomposition kernel and by the single-launch W4A16 decode GEMM.
#pragma once
#include "msd_common.hpp"

namespace msd {

// Exponent e of alpha = 2^e for a block with max-abs mb: smallest e with mb <= hi * 2^e, read off
// the fp32 fields (hi in [1, 2) given by its mantissa field: 1.859375 is 0x6E0000, 1.75 is
// 0x600000); clamped to [-123, 127].
__device__ __forceinline__ int mx_alpha_exponent(float mb, uint32_t hi_mant) {
  const uint32_t u = __float_as_uint(mb);
  int e = (int)(u >> 23) - 127;
  if ((u & 0x7FFFFFu) > hi_mant) e += 1;
  return min(max(e, -123), 127);
}

__device__ __forceinline__ float pow2f(int e) {  // e in [-126, 127]
  return __uint_as_float((uint32_t)(e + 127) << 23);
}

// 32 BF16 values of one block -> integer grid codes k1, k2 (value k/4) and exponent e.
// beta = alpha / 2^shift (shift 4 in Alg. 2).
__device__ __forceinline__ int mx_block_codes(const uint32_t (&w)[16], int (&k1)[32], int (&k2)[32],
                                              uint32_t hi_mant, int shift) {
  float mb = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    mb = fmaxf(mb, fabsf(__uint_as_float(w[i] << 16)));
    mb = fmaxf(mb, fabsf(__uint_as_float(w[i] & 0xFFFF0000u)));
  }
  const int e = mx_alpha_exponent(mb, hi_mant);
  const float up = pow2f(2 - e);    // 4/alpha
  const float down = pow2f(e - 2);  // alpha/4
  const float up2 = pow2f(shift);   // alpha/beta
#pragma unroll
  for (int i = 0; i < 32; ++i) {
    const float x = (i & 1) ? __uint_as_float(w[i >> 1] & 0xFFFF0000u) : __uint_as_float(w[i >> 1] << 16);
    const float a = fminf(fmaxf(rintf(x * up), -7.f), 7.f);
    const float r = __fmaf_rn(-a, down, x);  // exact
    const float b = fminf(fmaxf(rintf(r * up * up2), -7.f), 7.f);
    k1[i] = (int)a;
    k2[i] = (int)b;
  }
  return e;
}

// Same decomposition, packed on the fly: 32 BF16 values -> the FP6-E2M3 operands of both
// components (6 dwords each, element i at bits [6i, 6i+6)) and the exponent e.  Keeps no
// 32-element code arrays alive (the GEMM kernels that decompose in place are register-bound).
__device__ __forceinline__ int mx_block_pack_fp6(const uint32_t (&w)[16], uint32_t (&p1)[6], uint32_t (&p2)[6],
                                                 uint32_t hi_mant, int shift) {
  float mb = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    mb = fmaxf(mb, fabsf(__uint_as_float(w[i] << 16)));
    mb = fmaxf(mb, fabsf(__uint_as_float(w[i] & 0xFFFF0000u)));
  }
  const int e = mx_alpha_exponent(mb, hi_mant);
  const float up = pow2f(2 - e);    // 4/alpha
  const float down = pow2f(e - 2);  // alpha/4
  const float up2 = pow2f(shift);   // alpha/beta
#pragma unroll
  for (int h = 0; h < 2; ++h) {  // 16 codes -> 96 bits -> 3 dwords per component
    uint64_t lo1 = 0, lo2 = 0;
    uint32_t hi1 = 0, hi2 = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int idx = h * 16 + i;
      const float x = (idx & 1) ? __uint_as_float(w[idx >> 1] & 0xFFFF0000u) : __uint_as_float(w[idx >> 1] << 16);
      const float a = fminf(fmaxf(rintf(x * up), -7.f), 7.f);
      const float r = __fmaf_rn(-a, down, x);  // exact
      const float b = fminf(fmaxf(rintf(r * up * up2), -7.f), 7.f);
      const int ka = (int)a, kb = (int)b;
      const uint64_t c1 = ka < 0 ? (32u | (uint32_t)(-2 * ka)) : (uint32_t)(2 * ka);
      const uint64_t c2 = kb < 0 ? (32u | (uint32_t)(-2 * kb)) : (uint32_t)(2 * kb);
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

__device__ __forceinline__ uint32_t nibble4(int k) {  // sign-magnitude, -0 -> +0
  return k < 0 ? (8u | (uint32_t)(-k)) : (uint32_t)k;
}
__device__ __forceinline__ uint32_t e2m3_code(int k) {  // value k/4 as FP6 E2M3: magnitude field 2|k|
  return k < 0 ? (32u | (uint32_t)(-2 * k)) : (uint32_t)(2 * k);
}

// Pack 32 six-bit codes into 6 dwords, element i at bits [6i, 6i+6).
__device__ __forceinline__ void pack_fp6(const int (&k)[32], uint32_t (&out)[6]) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {  // 16 codes -> 96 bits -> 3 dwords
    uint64_t lo = 0;             // bits 0..63
    uint32_t hi = 0;             // bits 64..95
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const uint64_t c = e2m3_code(k[h * 16 + i]);
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
