// Shared device/host helpers of the gfx950 MSD library (not shared with the CPU oracle).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "msd.h"

namespace msd {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef short v8s __attribute__((ext_vector_type(8)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

constexpr int kWave = 64;

// error bookkeeping (host)
extern thread_local int g_last_hip_error;
inline int hip_fail(hipError_t e) {
  g_last_hip_error = (int)e;
  return MSD_ERR_HIP;
}
#define MSD_HIP_CHECK(expr)                          \
  do {                                               \
    hipError_t e__ = (expr);                         \
    if (e__ != hipSuccess) return msd::hip_fail(e__); \
  } while (0)
#define MSD_LAUNCH_CHECK() MSD_HIP_CHECK(hipGetLastError())

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- device helpers ------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// fp32 -> BF16 bits, round-to-nearest-even (finite inputs)
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Parameterisation of the two-pass MXFP4 decomposition (paper Sec. 3.3): alpha = 2^e with e the
// smallest exponent such that max|block| <= hi * 2^(e + ebias), hi in [1, 2) given by its fp32
// mantissa field; beta = alpha / 2^shift.  (1.859375, 4) is Alg. 2; the design-evolution table's
// earlier parameterisations are v1 = (1.75, 3) and v2 = (1.75, 4).  e2m1 = 1 is the ablation with
// both components on the MX FP4 element grid {0, .5, 1, 1.5, 2, 3, 4, 6} instead of the paper's
// uniform grid {k/4}: max|block| <= 6 alpha (hi = 1.5, ebias = 2), beta = alpha / 4.
struct MxVariant {
  uint32_t hi_mant = 0x6E0000u;  // 1.859375; 1.75 is 0x600000, 1.5 is 0x400000
  int shift = 4;
  int ebias = 0;
  int e2m1 = 0;
};

// Rotate within the 16-lane DPP row of a lane (lanes sharing lane/16): a cross-lane move on the vector
// ALU, no LDS round trip.
template <int N>
__device__ __forceinline__ float row16_ror(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x120 + N, 0xF, 0xF, false));
}
// Maximum over the 64 lanes of a full wave, returned in every lane: four rotate-and-max steps inside
// the rows, then the four row results through scalar registers.
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, row16_ror<8>(v));
  v = fmaxf(v, row16_ror<4>(v));
  v = fmaxf(v, row16_ror<2>(v));
  v = fmaxf(v, row16_ror<1>(v));
  const int b = __float_as_int(v);
  const float r0 = __int_as_float(__builtin_amdgcn_readlane(b, 0));
  const float r1 = __int_as_float(__builtin_amdgcn_readlane(b, 16));
  const float r2 = __int_as_float(__builtin_amdgcn_readlane(b, 32));
  const float r3 = __int_as_float(__builtin_amdgcn_readlane(b, 48));
  return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}

// One step of the two-pass INT8 decomposition (paper Sec. 3.2): given alpha, beta (already
// rounded fp32 quotients) produce the two codes of x.  Correctly rounded division,
// round-half-to-even, fused residual.
__device__ __forceinline__ void int8_codes(float x, float alpha, float beta, int& c1, int& c2) {
  float t = __fdiv_rn(x, alpha);
  float q = fminf(fmaxf(rintf(t), -128.f), 127.f);
  float r = __fmaf_rn(-alpha, q, x);
  float u = __fdiv_rn(r, beta);
  float p = fminf(fmaxf(rintf(u), -128.f), 127.f);
  c1 = (int)q;
  c2 = (int)p;
}

}  // namespace msd
