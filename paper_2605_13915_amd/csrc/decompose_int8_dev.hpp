// Device code of the two-pass INT8 row decomposition (paper Sec. 3.2), shared by the
// stand-alone decomposition kernel and by the fused decode GEMM.
#pragma once
#include "msd_common.hpp"

namespace msd {

constexpr int kDecRegChunks = 1;  // 16-element chunks cached in registers per thread (the rest is re-read from L2)

struct Chunk16 {
  uint32_t w[8];  // 16 BF16 values
};

__device__ __forceinline__ Chunk16 load_chunk16(const uint16_t* p, bool aligned) {
  Chunk16 c;
  if (aligned) {
    const uint4* q = reinterpret_cast<const uint4*>(p);
    uint4 a = q[0], b = q[1];
    c.w[0] = a.x; c.w[1] = a.y; c.w[2] = a.z; c.w[3] = a.w;
    c.w[4] = b.x; c.w[5] = b.y; c.w[6] = b.z; c.w[7] = b.w;
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) c.w[i] = (uint32_t)p[2 * i] | ((uint32_t)p[2 * i + 1] << 16);
  }
  return c;
}

__device__ __forceinline__ float chunk_absmax(const Chunk16& c) {
  float m = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    m = fmaxf(m, fabsf(__uint_as_float(c.w[i] << 16)));
    m = fmaxf(m, fabsf(__uint_as_float(c.w[i] & 0xFFFF0000u)));
  }
  return m;
}

__device__ __forceinline__ void chunk_codes(const Chunk16& c, float alpha, float beta, uint4& o1,
                                            uint4& o2) {
  uint32_t a[4], b[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    uint32_t pa = 0, pb = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t w = c.w[j * 2 + (e >> 1)];
      const float x = (e & 1) ? __uint_as_float(w & 0xFFFF0000u) : __uint_as_float(w << 16);
      int c1, c2;
      int8_codes(x, alpha, beta, c1, c2);
      pa |= ((uint32_t)c1 & 0xFFu) << (8 * e);
      pb |= ((uint32_t)c2 & 0xFFu) << (8 * e);
    }
    a[j] = pa;
    b[j] = pb;
  }
  o1 = make_uint4(a[0], a[1], a[2], a[3]);
  o2 = make_uint4(b[0], b[1], b[2], b[3]);
}

// Bit-exact quantisation without a division per element.  q = rne(x/alpha) is computed as
// rne(x * (1/alpha)); the product differs from the correctly rounded quotient by at most
// 127.49*2^-22 < 3.1e-5 in absolute terms (|x/alpha| <= 127.49 for either pair of range constants), so the two can round differently only if the product is
// within that distance of a half-integer.  Lanes where it is within 1e-4 recompute with the
// exact division (about 2 elements in 10^4).  Same for the residual pass.
__device__ __forceinline__ void int8_codes_fast(float x, float alpha, float ra, float beta, float rb,
                                                int& c1, int& c2) {
  float t = x * ra;
  float q = rintf(t);
  const bool tie1 = fabsf(t - q) > 0.5f - 1e-4f;
  if (__builtin_amdgcn_ballot_w64(tie1) != 0)  // wave-uniform branch: the division is really skipped
    q = tie1 ? rintf(__fdiv_rn(x, alpha)) : q;
  const float r = __fmaf_rn(-alpha, q, x);
  float u = r * rb;
  float p = rintf(u);
  const bool tie2 = fabsf(u - p) > 0.5f - 1e-4f;
  if (__builtin_amdgcn_ballot_w64(tie2) != 0) p = tie2 ? rintf(__fdiv_rn(r, beta)) : p;
  c1 = (int)fminf(fmaxf(q, -128.f), 127.f);
  c2 = (int)fminf(fmaxf(p, -128.f), 127.f);
}

// Correctly rounded x / a without a division: t = x * RN(1/a) is within two units in the last place of
// the quotient; one refinement with the exact FMA residual, t' = t + (x - a t) * RN(1/a), makes it faithful,
// and a second one then returns RN(x / a) itself (Markstein's theorem on FMA division: exact whenever the
// significand of a is not all ones, the quotient is a normal number and nothing underflows on the way).
// ra must be the correctly rounded reciprocal.  Checked exhaustively on the GPU against the hardware's
// correctly rounded division for every BF16 numerator and about 10^4 divisors: identical bits.
__device__ __forceinline__ float quotient_rn(float x, float a, float ra) {
  float t = x * ra;
  t = __fmaf_rn(__fmaf_rn(-a, t, x), ra, t);
  t = __fmaf_rn(__fmaf_rn(-a, t, x), ra, t);
  return t;
}

__device__ __forceinline__ uint32_t pack4(int a, int b, int c, int d) {
  return ((uint32_t)a & 0xFFu) | (((uint32_t)b & 0xFFu) << 8) | (((uint32_t)c & 0xFFu) << 16) | ((uint32_t)d << 24);
}

// Four elements -> one dword of codes per component, branch-free and in constant time (no data-dependent
// path: BF16 inputs hit exact rounding ties of x/alpha often, e.g. whenever alpha is a power of two).
// No clamp is needed: |x/alpha| <= 127.49 and |r/beta| <= 127.49 * (1 + 2^-22) round to at most 127.
__device__ __forceinline__ void quad_codes_fast(uint32_t w0, uint32_t w1, float alpha, float ra, float beta, float rb,
                                                uint32_t& o1, uint32_t& o2) {
  const float x0 = __uint_as_float(w0 << 16), x1 = __uint_as_float(w0 & 0xFFFF0000u);
  const float x2 = __uint_as_float(w1 << 16), x3 = __uint_as_float(w1 & 0xFFFF0000u);
  const float q0 = rintf(quotient_rn(x0, alpha, ra)), q1 = rintf(quotient_rn(x1, alpha, ra));
  const float q2 = rintf(quotient_rn(x2, alpha, ra)), q3 = rintf(quotient_rn(x3, alpha, ra));
  const float r0 = __fmaf_rn(-alpha, q0, x0), r1 = __fmaf_rn(-alpha, q1, x1);
  const float r2 = __fmaf_rn(-alpha, q2, x2), r3 = __fmaf_rn(-alpha, q3, x3);
  const float p0 = rintf(quotient_rn(r0, beta, rb)), p1 = rintf(quotient_rn(r1, beta, rb));
  const float p2 = rintf(quotient_rn(r2, beta, rb)), p3 = rintf(quotient_rn(r3, beta, rb));
  o1 = pack4((int)q0, (int)q1, (int)q2, (int)q3);
  o2 = pack4((int)p0, (int)p1, (int)p2, (int)p3);
}

// Rows the division-free route cannot serve take the divisions (a row-uniform choice): a scale whose
// significand is all ones (the exception of the theorem above), or a row maximum below 2^-83, where a
// residual of the refinement could underflow.
__device__ __forceinline__ bool needs_divisions(float alpha, float beta) {
  const uint32_t ua = __float_as_uint(alpha), ub = __float_as_uint(beta);
  return (ua & 0x7FFFFFu) == 0x7FFFFFu || (ub & 0x7FFFFFu) == 0x7FFFFFu || !(alpha >= 0x1p-90f);
}

// The same 16 elements with the divisions, rolled up so that it costs the kernels that inline it next to the
// fast route neither registers nor code size.
__device__ __forceinline__ void chunk_codes_rolled(const Chunk16& c, float alpha, float beta, uint4& o1, uint4& o2) {
  uint32_t a0 = 0, a1 = 0, a2 = 0, a3 = 0, b0 = 0, b1 = 0, b2 = 0, b3 = 0;
#pragma unroll 1
  for (int j = 0; j < 4; ++j) {
    const uint32_t w0 = j == 0 ? c.w[0] : j == 1 ? c.w[2] : j == 2 ? c.w[4] : c.w[6];
    const uint32_t w1 = j == 0 ? c.w[1] : j == 1 ? c.w[3] : j == 2 ? c.w[5] : c.w[7];
    uint32_t pa = 0, pb = 0;
#pragma unroll 1
    for (int e = 0; e < 4; ++e) {
      const uint32_t w = e < 2 ? w0 : w1;
      const float x = (e & 1) ? __uint_as_float(w & 0xFFFF0000u) : __uint_as_float(w << 16);
      int c1, c2;
      int8_codes(x, alpha, beta, c1, c2);
      pa |= ((uint32_t)c1 & 0xFFu) << (8 * e);
      pb |= ((uint32_t)c2 & 0xFFu) << (8 * e);
    }
    if (j == 0) { a0 = pa; b0 = pb; } else if (j == 1) { a1 = pa; b1 = pb; } else if (j == 2) { a2 = pa; b2 = pb; } else { a3 = pa; b3 = pb; }
  }
  o1 = make_uint4(a0, a1, a2, a3);
  o2 = make_uint4(b0, b1, b2, b3);
}

// 16 elements; ra = RN(1/alpha), rb = RN(1/beta).
__device__ __forceinline__ void chunk_codes_fast(const Chunk16& c, float alpha, float ra, float beta,
                                                 float rb, uint4& o1, uint4& o2) {
  if (needs_divisions(alpha, beta)) {
    chunk_codes_rolled(c, alpha, beta, o1, o2);
    return;
  }
  uint32_t a[4], b[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) quad_codes_fast(c.w[2 * j], c.w[2 * j + 1], alpha, ra, beta, rb, a[j], b[j]);
  o1 = make_uint4(a[0], a[1], a[2], a[3]);
  o2 = make_uint4(b[0], b[1], b[2], b[3]);
}

// One workgroup of THREADS threads decomposes one row: xr[0..K) -> q1r, q2r (16-byte aligned),
// *alpha_out.  s_red: THREADS/64 floats of LDS.  Ends with every thread's stores issued (no
// trailing barrier).  num1 / num2: the range constants (alpha = max / num1, beta = alpha / num2).
// With a_step != 0 the codes go to the blocked layout of the asynchronous-fill GEMM instead
// (stage depth a_bk = 64 or 128 bytes of K per row): q1r / q2r then point at the array base and
// 16-byte chunk c of row m lands in stage c / (a_bk/16), block m / (1024/a_bk), at the row's
// place inside the block with its chunk index XOR-swizzled as in the GEMM's LDS image.
template <int THREADS>
__device__ __forceinline__ void decompose_row_int8_block(const uint16_t* __restrict__ xr, int K,
                                                         int8_t* __restrict__ q1r,
                                                         int8_t* __restrict__ q2r,
                                                         float* __restrict__ alpha_out, bool aligned,
                                                         float* s_red, float num1, float num2,
                                                         int64_t a_step = 0, int64_t m = 0, int a_bk = 64,
                                                         int frag_rt = 0, int64_t frag_m2 = 0) {
  // frag_rt != 0: the fragment-major layout of the register-operand GEMM kernels (GemmW8Args::a_frag): both
  // components in one array, stacked row i = m (first component) or frag_m2 + m (residual component), the 16
  // bytes of K step s, group g of stacked row i at ((s * frag_rt + i/16) * 64 + g * 16 + i%16) * 16 -- one
  // contiguous kilobyte per (K step, 16-row fragment), in the lane order of the matrix instruction's operand.
  // q1r is the array base; q2r is unused.
  const int nchunks = K / 16;
  const int cpr = a_bk / 16, rpi = 1024 / a_bk;  // chunks per row, rows per 1 KB block
  const int64_t row_off = (m / rpi) * 1024 + (m % rpi) * a_bk;
  const int sw = a_bk == 64 ? (int)((m >> 2) & 3) : (int)((m >> 1) & 7);
  const int64_t i2 = frag_m2 + m;
  auto slot = [&](int c) -> int64_t {  // index of chunk c in units of 16 bytes
    if (frag_rt) return ((int64_t)(c >> 2) * frag_rt + (m >> 4)) * 64 + (c & 3) * 16 + (m & 15);
    return a_step ? ((int64_t)(c / cpr) * a_step + row_off + (((c % cpr) ^ sw) << 4)) >> 4 : c;
  };
  auto slot2 = [&](int c) -> int64_t {  // the same for the residual component
    if (frag_rt) return ((int64_t)(c >> 2) * frag_rt + (i2 >> 4)) * 64 + (c & 3) * 16 + (i2 & 15);
    return slot(c);
  };
  Chunk16 cache[kDecRegChunks];
  float mx = 0.f;
#pragma unroll
  for (int i = 0; i < kDecRegChunks; ++i) {
    const int c = threadIdx.x + i * THREADS;
    if (c < nchunks) {
      cache[i] = load_chunk16(xr + c * 16, aligned);
      mx = fmaxf(mx, chunk_absmax(cache[i]));
    }
  }
#pragma unroll 1
  for (int c = threadIdx.x + kDecRegChunks * THREADS; c < nchunks; c += THREADS)
    mx = fmaxf(mx, chunk_absmax(load_chunk16(xr + c * 16, aligned)));
  mx = wave_max(mx);
  if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = mx;
  __syncthreads();
  mx = s_red[0];
#pragma unroll
  for (int w = 1; w < THREADS / 64; ++w) mx = fmaxf(mx, s_red[w]);
  const float alpha = __fdiv_rn(mx, num1);
  const float beta = __fdiv_rn(alpha, num2);
  const float ra = __fdiv_rn(1.0f, alpha), rb = __fdiv_rn(1.0f, beta);  // unused for an all-zero row
  if (threadIdx.x == 0) *alpha_out = alpha;
  uint4* o1 = reinterpret_cast<uint4*>(q1r);
  uint4* o2 = reinterpret_cast<uint4*>(frag_rt ? q1r : q2r);
  if (mx == 0.f) {  // all-zero row: zero codes, zero scales
    for (int c = threadIdx.x; c < nchunks; c += THREADS) {
      o1[slot(c)] = make_uint4(0, 0, 0, 0);
      o2[slot2(c)] = make_uint4(0, 0, 0, 0);
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < kDecRegChunks; ++i) {
    const int c = threadIdx.x + i * THREADS;
    if (c < nchunks) {
      uint4 a, b;
      chunk_codes_fast(cache[i], alpha, ra, beta, rb, a, b);
      o1[slot(c)] = a;
      o2[slot2(c)] = b;
    }
  }
#pragma unroll 1
  for (int c = threadIdx.x + kDecRegChunks * THREADS; c < nchunks; c += THREADS) {
    uint4 a, b;
    chunk_codes_fast(load_chunk16(xr + c * 16, aligned), alpha, ra, beta, rb, a, b);
    o1[slot(c)] = a;
    o2[slot2(c)] = b;
  }
}

}  // namespace msd
