/*
 * CPU oracle for Multi-Scale Dequant (MSD).  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct implementation of what the hot path computes,
 * written from the paper's equations and algorithms.  It shares no code, header,
 * table or helper with the HIP path and is never linked into the product library.
 * Only tests, the smoke check and the CPU-baseline leg of the benchmark call it.
 *
 * Conventions
 *   - BF16 values travel as raw uint16_t bit patterns (upper half of an IEEE fp32).
 *   - GEMM shapes are (M, K, N): M activation rows (paper's batch b), K contraction
 *     (paper's n), N output channels (paper's m).  W is stored [N][K], K contiguous,
 *     so y[M][N] = X . W^T   (Sec. 3.1, problem formulation).
 *   - All decomposition arithmetic is IEEE fp32 with round-to-nearest-even; build with
 *     -ffp-contract=off so that only the explicit fmaf() below fuses.
 *   - round() in the paper is taken as round-half-to-even.
 *   - The only parallelism is an OpenMP loop over independent activation rows /
 *     (batch, head) pairs; there is no blocking, fusion or reordering.
 *
 * Pin status (see tests/test_oracle_*.py): every function below is pinned by the
 * paper's theorems, closed forms, brute force on tiny inputs or an independently
 * written exact-rational implementation.  msd_oracle_attn_decode in per-token scale
 * mode (a reading: the paper states attention for per-channel scales only) is pinned
 * by reduction to the per-channel statement -- identical codes and output for uniform
 * power-of-two scales, exact equivalence of scaling s_K[t] and scaling the INT8 row
 * K[t] by a power of two -- next to the invariants and the fp64 truth.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define MSD_FMT_INT8 0
#define MSD_FMT_MXFP4 1
#define MSD_SCALE_PER_TOKEN 0
#define MSD_SCALE_PER_CHANNEL 1

/* ---------- small helpers ------------------------------------------------ */

static float bf16_to_f32(uint16_t h) {
  uint32_t u = ((uint32_t)h) << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

/* fp32 -> bf16, round-to-nearest-even (finite inputs). */
static uint16_t f32_to_bf16_rne(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7FFFu + lsb;
  return (uint16_t)(u >> 16);
}

static int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

/* round-half-to-even of an fp32 value to an int (|v| small). */
static int rne_i(float v) { return (int)nearbyintf(v); }

/* ---------- two-pass INT8 decomposition (Sec. 3.2, Eqs. alpha, x1, r, beta, x2;
 *            Alg. 1 steps 1-5) ------------------------------------------------
 * num1/num2 are the two range constants: 127 and 254 in the paper's main variant,
 * 127.49 and 254.98 in the "fractional scaling" refinement of Sec. 3.3.
 * One row x[0..K): returns alpha, beta and the two INT8 code vectors.
 */
static void decompose_row_int8(const uint16_t* x, int64_t K, float num1, float num2, int8_t* q1,
                               int8_t* q2, float* alpha_out, float* beta_out) {
  float mx = 0.0f;
  for (int64_t k = 0; k < K; ++k) {
    float a = fabsf(bf16_to_f32(x[k]));
    if (a > mx) mx = a;
  }
  if (mx == 0.0f) { /* all-zero row: scales and codes are zero */
    memset(q1, 0, (size_t)K);
    memset(q2, 0, (size_t)K);
    *alpha_out = 0.0f;
    *beta_out = 0.0f;
    return;
  }
  const float alpha = mx / num1;   /* alpha = ||x||_inf / 127 */
  const float beta = alpha / num2; /* beta  = alpha / 254     */
  for (int64_t k = 0; k < K; ++k) {
    const float xv = bf16_to_f32(x[k]);
    const int c1 = clampi(rne_i(xv / alpha), -128, 127);
    const float r = fmaf(-alpha, (float)c1, xv); /* r = x - alpha*x1, one rounding */
    const int c2 = clampi(rne_i(r / beta), -128, 127);
    q1[k] = (int8_t)c1;
    q2[k] = (int8_t)c2;
  }
  *alpha_out = alpha;
  *beta_out = beta;
}

void msd_oracle_decompose_int8(const uint16_t* x_bf16, int64_t M, int64_t K, int64_t ldx,
                               int fractional, int8_t* q1, int8_t* q2, float* alpha,
                               float* beta) {
  const float n1 = fractional ? 127.49f : 127.0f;
  const float n2 = fractional ? 254.98f : 254.0f;
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    decompose_row_int8(x_bf16 + m * ldx, K, n1, n2, q1 + m * K, q2 + m * K, alpha + m, beta + m);
}

/* ---------- W8A16 MSD linear layer (Alg. 1; Sec. 3.1 last equation) -------
 * acc1 = q1 . W^T, acc2 = q2 . W^T in exact integers, then
 * y = s_W (.) (alpha*acc1 + beta*acc2), evaluated in fp64 and rounded once.
 * Optional taps (may be NULL): q1,q2 [M][K], alpha,beta [M], acc1,acc2 [M][N] (int32),
 * overflow: set to 1 if any int64 accumulator leaves the int32 range.
 * out_bf16 != 0: y is uint16_t BF16 (RNE of the fp32 result), else float.
 */
void msd_oracle_gemm_w8a16(const uint16_t* x_bf16, int64_t M, int64_t K, int64_t ldx,
                           const int8_t* W, const float* w_scale, int64_t N, int fractional,
                           void* y, int out_bf16, int64_t ldy, int8_t* tap_q1, int8_t* tap_q2,
                           float* tap_alpha, float* tap_beta, int32_t* tap_acc1,
                           int32_t* tap_acc2, int* overflow) {
  const float n1 = fractional ? 127.49f : 127.0f;
  const float n2 = fractional ? 254.98f : 254.0f;
  int ovf = 0;
#pragma omp parallel for schedule(static) reduction(| : ovf)
  for (int64_t m = 0; m < M; ++m) {
    int8_t* q1 = (int8_t*)malloc((size_t)K);
    int8_t* q2 = (int8_t*)malloc((size_t)K);
    float alpha, beta;
    decompose_row_int8(x_bf16 + m * ldx, K, n1, n2, q1, q2, &alpha, &beta);
    if (tap_q1) memcpy(tap_q1 + m * K, q1, (size_t)K);
    if (tap_q2) memcpy(tap_q2 + m * K, q2, (size_t)K);
    if (tap_alpha) tap_alpha[m] = alpha;
    if (tap_beta) tap_beta[m] = beta;
    for (int64_t n = 0; n < N; ++n) {
      const int8_t* w = W + n * K;
      int64_t a1 = 0, a2 = 0;
      for (int64_t k = 0; k < K; ++k) {
        a1 += (int64_t)q1[k] * (int64_t)w[k];
        a2 += (int64_t)q2[k] * (int64_t)w[k];
      }
      if (a1 > INT32_MAX || a1 < INT32_MIN || a2 > INT32_MAX || a2 < INT32_MIN) ovf |= 1;
      if (tap_acc1) tap_acc1[m * N + n] = (int32_t)a1;
      if (tap_acc2) tap_acc2[m * N + n] = (int32_t)a2;
      const double v = (double)w_scale[n] * ((double)alpha * (double)a1 + (double)beta * (double)a2);
      const float vf = (float)v;
      if (out_bf16)
        ((uint16_t*)y)[m * ldy + n] = f32_to_bf16_rne(vf);
      else
        ((float*)y)[m * ldy + n] = vf;
    }
    free(q1);
    free(q2);
  }
  if (overflow) *overflow = ovf;
}

/* fp64 truth for the linear layer: y = X . (s_W (.) W)^T with no activation quantisation. */
void msd_oracle_truth_gemm_w8(const uint16_t* x_bf16, int64_t M, int64_t K, int64_t ldx,
                              const int8_t* W, const float* w_scale, int64_t N, double* y) {
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      double s = 0.0;
      for (int64_t k = 0; k < K; ++k)
        s += (double)bf16_to_f32(x_bf16[m * ldx + k]) * (double)W[n * K + k];
      y[m * N + n] = s * (double)w_scale[n];
    }
}

/* Dequantisation baseline the paper compares against (Sec. 3.1 first equation, Sec. 6.1):
 * W is lifted to BF16 as bf16(s_W[n] * W[n][k]), then BF16 x BF16 products are summed.
 * Products of two BF16 values are exact in fp32/fp64; the sum is taken in fp64. */
void msd_oracle_dequant_gemm_w8a16(const uint16_t* x_bf16, int64_t M, int64_t K, int64_t ldx,
                                   const int8_t* W, const float* w_scale, int64_t N, float* y) {
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      double s = 0.0;
      for (int64_t k = 0; k < K; ++k) {
        const float wd = bf16_to_f32(f32_to_bf16_rne(w_scale[n] * (float)W[n * K + k]));
        s += (double)bf16_to_f32(x_bf16[m * ldx + k]) * (double)wd;
      }
      y[m * N + n] = (float)s;
    }
}

/* ---------- two-pass MXFP4 decomposition (Sec. 3.2.1, Alg. 2) --------------
 * Per 32-element block.  All arithmetic is exact (powers of two and small integers).
 *   alpha = 2^e,  e = ceil(log2(M_b / hi))   with hi = 1.859375 (v3) or 1.75 (v1, v2)
 *   q1 = nearest point of the uniform grid {k/4, |k| <= 7} to x/alpha (saturating)
 *   r  = x - alpha*q1
 *   beta = alpha / 2^shift   with shift = 4 (v2, v3) or 3 (v1)
 *   q2 = nearest grid point to r/beta (saturating)
 * Codes are 4-bit sign-magnitude nibbles (bit 3 = sign, bits 2..0 = k, value k/4),
 * -0 stored as +0; two per byte, low nibble = even k.  Scale byte = e + 127 (E8M0);
 * e is clamped to [-123, 127] so that beta's byte e + 127 - shift is a valid E8M0.
 * An all-zero block gets e = -123 and zero codes.
 * variant 4 is the E2M1-grid ablation described further down (codes are then OCP E2M1 nibbles,
 * shift = 2).
 */
static int mx_alpha_exp(float mb, int variant) {
  if (mb == 0.0f) return -123;
  int ex;
  const float fr = frexpf(mb, &ex); /* mb = fr * 2^ex, fr in [0.5, 1) */
  const float f = 2.0f * fr;        /* in [1, 2), exact */
  const int E = ex - 1;
  if (variant == 4) { /* E2M1 grid: smallest e with mb <= 6 * 2^e = 1.5 * 2^(e+2) */
    const int e4 = (f <= 1.5f) ? E - 2 : E - 1;
    return clampi(e4, -123, 127);
  }
  const float hi = (variant == 3) ? 1.859375f : 1.75f;
  int e = (f <= hi) ? E : E + 1; /* smallest e with mb <= hi * 2^e */
  return clampi(e, -123, 127);
}

/* ---------- ablation: both components on the OCP E2M1 grid (variant 4) -------------------
 * The paper's components live on the uniform grid {k/4}; Sec. 2.2 / Sec. 3.2.1 attribute the format to
 * the MX specification, whose FP4 element is E2M1 with magnitudes {0, .5, 1, 1.5, 2, 3, 4, 6}.  This
 * variant runs the same two passes on that grid, so that a native FP4 x FP4 product could consume the
 * components:  alpha = 2^e with e the smallest exponent such that M_b <= 6 alpha;  q1 = nearest E2M1
 * value to x/alpha (ties to the even code);  r = x - alpha q1 (exact);  beta = alpha / 4;  q2 = nearest
 * E2M1 value to r/beta.  |r| <= alpha (half the widest gap, 2, at the top of the range), hence
 * |r/beta| <= 4: the second pass never saturates, and its error is at most half a gap of 1 at that
 * magnitude: |x - (alpha q1 + beta q2)| <= beta/2 = alpha/8, against alpha/64 on the uniform grid.
 * Codes are OCP E2M1 nibbles (bit 3 sign, bits 2..1 exponent, bit 0 mantissa), -0 stored as +0.
 */
static const int kE2m1Halves[8] = {0, 1, 2, 3, 4, 6, 8, 12}; /* magnitude code -> value in halves */

/* nearest E2M1 magnitude code to v >= 0 (v exact); ties go to the even code; saturates at 6 */
static int e2m1_nearest_code(float v) {
  int best = 0;
  float bd = v; /* distance to code 0 */
  for (int c = 1; c < 8; ++c) {
    const float d = fabsf(v - 0.5f * (float)kE2m1Halves[c]);
    if (d < bd || (d == bd && (c & 1) == 0)) {
      best = c;
      bd = d;
    }
  }
  return best;
}

static uint8_t e2m1_nibble(float scaled) { /* scaled = value / scale, exact */
  const int c = e2m1_nearest_code(fabsf(scaled));
  return (uint8_t)(c == 0 ? 0 : ((scaled < 0.0f ? 8 : 0) | c));
}
static float e2m1_value(uint8_t nib) { return (nib & 8 ? -0.5f : 0.5f) * (float)kE2m1Halves[nib & 7]; }

static int grid_code(float scaled) { /* scaled = 4 * value / scale, exact */
  return clampi(rne_i(scaled), -7, 7);
}

static uint8_t nibble_of(int k) { return k == 0 ? 0 : (uint8_t)((k < 0 ? 8 : 0) | abs(k)); }

void msd_oracle_decompose_mxfp4(const uint16_t* x_bf16, int64_t M, int64_t K, int64_t ldx,
                                int variant, uint8_t* q1 /*[M][K/2]*/, uint8_t* q2 /*[M][K/2]*/,
                                uint8_t* e8m0_alpha /*[M][K/32]*/) {
  const int shift = (variant == 1) ? 3 : 4;
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m) {
    for (int64_t b = 0; b < K / 32; ++b) {
      const uint16_t* xb = x_bf16 + m * ldx + b * 32;
      float mb = 0.0f;
      for (int i = 0; i < 32; ++i) {
        float a = fabsf(bf16_to_f32(xb[i]));
        if (a > mb) mb = a;
      }
      const int e = mx_alpha_exp(mb, variant);
      e8m0_alpha[m * (K / 32) + b] = (uint8_t)(e + 127);
      for (int i = 0; i < 32; i += 2) {
        uint8_t n1[2], n2[2];
        for (int j = 0; j < 2; ++j) {
          const float xv = bf16_to_f32(xb[i + j]);
          if (variant == 4) {
            n1[j] = e2m1_nibble(ldexpf(xv, -e));                 /* x/alpha */
            const float r = xv - ldexpf(e2m1_value(n1[j]), e);    /* x - alpha*q1, exact */
            n2[j] = e2m1_nibble(ldexpf(r, 2 - e));                /* r/beta, beta = alpha/4 */
            continue;
          }
          const int k1 = grid_code(ldexpf(xv, 2 - e));      /* 4*x/alpha */
          const float r = xv - ldexpf((float)k1, e - 2);    /* x - alpha*k1/4, exact */
          const int k2 = grid_code(ldexpf(r, 2 - e + shift)); /* 4*r/beta */
          n1[j] = nibble_of(k1);
          n2[j] = nibble_of(k2);
        }
        q1[m * (K / 2) + b * 16 + i / 2] = (uint8_t)(n1[0] | (n1[1] << 4));
        q2[m * (K / 2) + b * 16 + i / 2] = (uint8_t)(n2[0] | (n2[1] << 4));
      }
    }
  }
}

/* value of a sign-magnitude activation nibble in quarters (integer k, value k/4) */
static int act_nibble_quarters(uint8_t nib) { return (nib & 8) ? -(int)(nib & 7) : (int)(nib & 7); }

/* value of an OCP E2M1 weight nibble in halves (integer h, value h/2):
 * magnitudes {0, .5, 1, 1.5, 2, 3, 4, 6}. */
static int e2m1_halves(uint8_t nib) {
  static const int mag[8] = {0, 1, 2, 3, 4, 6, 8, 12};
  return (nib & 8) ? -mag[nib & 7] : mag[nib & 7];
}

/* ---------- W4A16 MSD GEMM (Sec. 3.4.1; Alg. 2 feeding two block-scaled FP4 GEMMs) ----
 * y[m][n] = sum_b 2^(eW[n][b]-127) * ( 2^e_b * <q1_b, w_b> + 2^(e_b-shift) * <q2_b, w_b> ).
 * Each block dot product is an exact integer in units of 1/8; the sum over blocks is
 * taken in fp64 and rounded once to fp32 (or to BF16 after that).
 * Taps (nullable): q1,q2 nibble-packed [M][K/2], e8m0 [M][K/32].
 */
void msd_oracle_gemm_w4a16(const uint16_t* x_bf16, int64_t M, int64_t K, int64_t ldx,
                           const uint8_t* W_fp4 /*[N][K/2]*/, const uint8_t* W_e8m0 /*[N][K/32]*/,
                           int64_t N, int variant, void* y, int out_bf16, int64_t ldy,
                           uint8_t* tap_q1, uint8_t* tap_q2, uint8_t* tap_e8m0) {
  /* beta = alpha / 2^shift; the components are k/4 (unit 1/4) or, for the E2M1-grid ablation, h/2 */
  const int shift = (variant == 1) ? 3 : (variant == 4) ? 2 : 4;
  const int unit = (variant == 4) ? 2 : 3; /* block dots are integers in units of 2^-unit */
  const int64_t KB = K / 32;
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m) {
    uint8_t* q1 = (uint8_t*)malloc((size_t)(K / 2));
    uint8_t* q2 = (uint8_t*)malloc((size_t)(K / 2));
    uint8_t* ea = (uint8_t*)malloc((size_t)KB);
    msd_oracle_decompose_mxfp4(x_bf16 + m * ldx, 1, K, K, variant, q1, q2, ea);
    if (tap_q1) memcpy(tap_q1 + m * (K / 2), q1, (size_t)(K / 2));
    if (tap_q2) memcpy(tap_q2 + m * (K / 2), q2, (size_t)(K / 2));
    if (tap_e8m0) memcpy(tap_e8m0 + m * KB, ea, (size_t)KB);
    for (int64_t n = 0; n < N; ++n) {
      double s = 0.0;
      for (int64_t b = 0; b < KB; ++b) {
        int64_t d1 = 0, d2 = 0; /* in units of (1/4)*(1/2) = 1/8, or (1/2)*(1/2) = 1/4 on the E2M1 grid */
        for (int i = 0; i < 32; ++i) {
          const int64_t kk = b * 32 + i;
          const uint8_t wb = W_fp4[n * (K / 2) + kk / 2];
          const int w = e2m1_halves((kk & 1) ? (wb >> 4) : (wb & 15));
          const uint8_t a1 = q1[kk / 2], a2 = q2[kk / 2];
          const uint8_t c1 = (kk & 1) ? (a1 >> 4) : (a1 & 15), c2 = (kk & 1) ? (a2 >> 4) : (a2 & 15);
          d1 += (int64_t)(variant == 4 ? e2m1_halves(c1) : act_nibble_quarters(c1)) * w;
          d2 += (int64_t)(variant == 4 ? e2m1_halves(c2) : act_nibble_quarters(c2)) * w;
        }
        const int ew = (int)W_e8m0[n * KB + b] - 127;
        const int e = (int)ea[b] - 127;
        s += ldexp((double)d1, ew + e - unit) + ldexp((double)d2, ew + e - shift - unit);
      }
      const float vf = (float)s;
      if (out_bf16)
        ((uint16_t*)y)[m * ldy + n] = f32_to_bf16_rne(vf);
      else
        ((float*)y)[m * ldy + n] = vf;
    }
    free(q1);
    free(q2);
    free(ea);
  }
}

/* fp64 truth for W4A16: y = X . dequant(W)^T, activations not quantised. */
void msd_oracle_truth_gemm_w4(const uint16_t* x_bf16, int64_t M, int64_t K, int64_t ldx,
                              const uint8_t* W_fp4, const uint8_t* W_e8m0, int64_t N, double* y) {
  const int64_t KB = K / 32;
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      double s = 0.0;
      for (int64_t kk = 0; kk < K; ++kk) {
        const uint8_t wb = W_fp4[n * (K / 2) + kk / 2];
        const int w = e2m1_halves((kk & 1) ? (wb >> 4) : (wb & 15));
        const int ew = (int)W_e8m0[n * KB + kk / 32] - 127;
        s += (double)bf16_to_f32(x_bf16[m * ldx + kk]) * ldexp((double)w, ew - 1);
      }
      y[m * N + n] = s;
    }
}

/* ---------- MSD attention, one decode step (Sec. 4.2, Alg. 3), untiled ------
 * q [B][Hq][d] BF16;  K,V [B][Hkv][L][d] INT8;  query head hq reads KV head hq / (Hq/Hkv).
 * scale_mode PER_CHANNEL (the paper's statement): k_scale, v_scale are [Hkv][d];
 *     Q~ = Q (.) s_K is decomposed; S = (aQ*S1 + bQ*S2)/sqrt(d); P = exp(S - max S);
 *     P is decomposed with the constant alpha_P = 1/127; O = (aP*O1 + bP*O2) (.) s_V / l.
 * scale_mode PER_TOKEN (scales [B][Hkv][L]): Q itself is decomposed and s_K[t] multiplies
 *     column t of S; P~_t = P_t * s_V[t] is decomposed with alpha_P = max_t s_V[t] / 127
 *     (a bound on P~ that needs no reduction over P, as in the paper's constant-scale
 *     argument); O = (aP*O1 + bP*O2) / l.
 * l = sum_t P_t uses the undecomposed P (Alg. 3, last step).  kv_len[b] (nullable) gives
 * the number of valid tokens per batch entry; values outside [0, L] are clamped to it.
 * out: fp32 [B][Hq][d].  Taps (nullable): q codes [B][Hq][d] x2, alpha_q [B][Hq],
 * s1,s2 int32 [B][Hq][L], P float [B][Hq][L], p1,p2 int8 [B][Hq][L].
 */
/* The general form behind both entry points: query / key rows of d channels, value rows of dv
 * channels, key row t of KV head g at Kc + ((b*Hkv + g)*L + t)*ldk (values likewise with ldv), scores
 * multiplied by sm_scale.  Per-channel scales: k_scale [Hkv][d], v_scale [Hkv][dv]. */
/* Nearest binary16 (FP16) value of x, ties to even, returned as a float; |x| < 65520.  binary16 keeps 11
 * significant bits down to 2^-14 and a fixed quantum of 2^-24 below.  A sum, difference or product of two
 * binary16 values computed in fp32 and rounded with this function is the correctly rounded binary16 result
 * (fp32 carries 24 >= 2*11 + 2 bits, so the intermediate rounding is harmless). */
static float f16_rne(float x) {
  if (x == 0.0f || !isfinite(x)) return x;
  int e;
  (void)frexpf(fabsf(x), &e); /* |x| = m * 2^e with m in [0.5, 1) */
  int q = e - 11;             /* exponent of the last kept bit */
  if (q < -24) q = -24;
  return copysignf(ldexpf(rintf(ldexpf(fabsf(x), -q)), q), x);
}

/* Low-precision variant of the attention arithmetic (Sec. 4.4, "optimisation opportunities": the decomposition
 * (round, clamp) and the S / O merging (scale, add) in 16-bit floating-point or integer arithmetic in place of
 * fp32).  The paper gives one sentence; the reading taken here (lowprec != 0):
 *   S merge    : alpha_Q S1 + beta_Q S2 = beta_Q (254 S1 + S2) exactly, so the merge is the exact integer
 *                z = 254 S1 + S2 (|z| < 2^30), ONE conversion to fp32 and ONE fp32 multiply by
 *                c_t = (beta_Q * sm_scale) * s_K[t] (both products in fp32).  Integer arithmetic replaces the
 *                scale-and-add; FP16 cannot hold S1 (up to 127*127*d).
 *   P codes    : v = P~ / alpha_P (in [0, 127]) is formed in fp32 as before, rounded ONCE to FP16 (ties to
 *                even), and both passes run in FP16: q1 = rne(v_h) via (v_h + 1536) - 1536 (FP16 quantum at
 *                1536 is 1), r = v_h - q1 (exact), q2 = rne(254 r) via the fused (254 r + 1536) - 1536: the
 *                product is exact inside the fused operation, so q2 is the round-half-even of the exact 254 r.
 *                No clamp can fire: v_h <= 127 and |r| <= 1/2 give |254 r| <= 127.
 *   O merge    : alpha_P O1 + beta_P O2 = beta_P (254 O1 + O2), the same identity (exact in this oracle, which
 *                carries O in fp64 either way).
 * Error of the decomposition, in units of alpha_P, for v in [0, 127]:
 *   |v - (q1 + q2/254)| <= |v - v_h| + |r - q2/254| <= 2^-11 v + 1/508,
 * the first term from the one FP16 rounding (relative 2^-11), the second from rne(254 r).  Against the fp32
 * form's 1/508 this adds a RELATIVE 2^-11: 32 times larger for the largest probabilities, equal for small
 * ones.  q1, r and q2 are exact functions of v_h. */
static void attn_decode_general(const uint16_t* q_bf16, const int8_t* Kc, int64_t ldk, const int8_t* Vc,
                                int64_t ldv, const float* k_scale, const float* v_scale, int scale_mode,
                                int B, int Hq, int Hkv, int d, int dv, double sm_scale, int lowprec,
                                const int32_t* kv_len, int64_t L, float* out, int8_t* tap_q1,
                                int8_t* tap_q2, float* tap_alpha_q, int32_t* tap_s1, int32_t* tap_s2,
                                float* tap_p, int8_t* tap_p1, int8_t* tap_p2) {
  const int G = Hq / Hkv;
  const double inv_sqrt_d = sm_scale;
#pragma omp parallel for schedule(dynamic)
  for (int bh = 0; bh < B * Hq; ++bh) {
    const int b = bh / Hq, hq = bh % Hq, g = hq / G;
    int64_t len = kv_len ? kv_len[b] : L;
    if (len > L) len = L; /* entries past the cache are read as the cache length (the library clamps likewise) */
    const int8_t* Kh = Kc + ((int64_t)(b * Hkv + g)) * L * ldk;
    const int8_t* Vh = Vc + ((int64_t)(b * Hkv + g)) * L * ldv;
    float* o = out + (int64_t)bh * dv;
    if (len <= 0) {
      for (int c = 0; c < dv; ++c) o[c] = 0.0f;
      continue;
    }
    /* steps 1-2: absorb s_K (per-channel mode) and decompose the query row */
    uint16_t* qt = (uint16_t*)malloc(sizeof(uint16_t) * (size_t)d);
    float* qf = (float*)malloc(sizeof(float) * (size_t)d);
    int8_t* q1 = (int8_t*)malloc((size_t)d);
    int8_t* q2 = (int8_t*)malloc((size_t)d);
    float aq, bq;
    if (scale_mode == MSD_SCALE_PER_CHANNEL) {
      /* Q~ is an fp32 vector, not BF16: decompose it with the same five steps */
      float mx = 0.0f;
      for (int c = 0; c < d; ++c) {
        qf[c] = bf16_to_f32(q_bf16[(int64_t)bh * d + c]) * k_scale[g * d + c];
        if (fabsf(qf[c]) > mx) mx = fabsf(qf[c]);
      }
      if (mx == 0.0f) {
        aq = bq = 0.0f;
        memset(q1, 0, (size_t)d);
        memset(q2, 0, (size_t)d);
      } else {
        aq = mx / 127.0f;
        bq = aq / 254.0f;
        for (int c = 0; c < d; ++c) {
          const int c1 = clampi(rne_i(qf[c] / aq), -128, 127);
          const float r = fmaf(-aq, (float)c1, qf[c]);
          q1[c] = (int8_t)c1;
          q2[c] = (int8_t)clampi(rne_i(r / bq), -128, 127);
        }
      }
    } else {
      for (int c = 0; c < d; ++c) qt[c] = q_bf16[(int64_t)bh * d + c];
      decompose_row_int8(qt, d, 127.0f, 254.0f, q1, q2, &aq, &bq);
    }
    if (tap_q1) memcpy(tap_q1 + (int64_t)bh * d, q1, (size_t)d);
    if (tap_q2) memcpy(tap_q2 + (int64_t)bh * d, q2, (size_t)d);
    if (tap_alpha_q) tap_alpha_q[bh] = aq;
    /* steps 3-5: S1, S2 integer GEMVs, merge */
    double* S = (double*)malloc(sizeof(double) * (size_t)len);
    float* P = (float*)malloc(sizeof(float) * (size_t)len);
    double smax = -INFINITY;
    for (int64_t t = 0; t < len; ++t) {
      int64_t s1 = 0, s2 = 0;
      for (int c = 0; c < d; ++c) {
        s1 += (int64_t)q1[c] * Kh[t * ldk + c];
        s2 += (int64_t)q2[c] * Kh[t * ldk + c];
      }
      if (tap_s1) tap_s1[(int64_t)bh * L + t] = (int32_t)s1;
      if (tap_s2) tap_s2[(int64_t)bh * L + t] = (int32_t)s2;
      double s;
      if (lowprec) { /* integer merge, one conversion, one fp32 multiply */
        const float zf = (float)(254 * s1 + s2);
        float c = bq * (float)inv_sqrt_d;
        if (scale_mode == MSD_SCALE_PER_TOKEN) c = c * k_scale[((int64_t)(b * Hkv + g)) * L + t];
        s = (double)(zf * c);
      } else {
        s = ((double)aq * (double)s1 + (double)bq * (double)s2) * inv_sqrt_d;
        if (scale_mode == MSD_SCALE_PER_TOKEN) s *= (double)k_scale[((int64_t)(b * Hkv + g)) * L + t];
      }
      S[t] = s;
      if (s > smax) smax = s;
    }
    /* steps 6-7: P = exp(S - m), l = sum P */
    double ell = 0.0;
    for (int64_t t = 0; t < len; ++t) {
      P[t] = (float)exp(S[t] - smax);
      ell += (double)P[t];
    }
    /* steps 8-9: decompose P with a scale that needs no reduction over P */
    float ap_num; /* alpha_P = ap_num / 127 */
    if (scale_mode == MSD_SCALE_PER_TOKEN) {
      ap_num = 0.0f;
      for (int64_t t = 0; t < len; ++t) {
        const float sv = v_scale[((int64_t)(b * Hkv + g)) * L + t];
        if (sv > ap_num) ap_num = sv;
      }
    } else {
      ap_num = 1.0f;
    }
    int8_t* p1 = (int8_t*)malloc((size_t)len);
    int8_t* p2 = (int8_t*)malloc((size_t)len);
    double ap, bp;
    if (lowprec) {
      float to_code; /* 1 / alpha_P */
      if (scale_mode == MSD_SCALE_PER_TOKEN) {
        const float apf = ap_num / 127.0f;
        ap = apf;
        bp = apf / 254.0f;
        to_code = ap_num > 0.0f ? 127.0f / ap_num : 0.0f;
      } else {
        ap = 1.0 / 127.0;
        bp = 1.0 / (127.0 * 254.0);
        to_code = 127.0f;
      }
      for (int64_t t = 0; t < len; ++t) {
        float v = P[t];
        if (scale_mode == MSD_SCALE_PER_TOKEN) v = v * v_scale[((int64_t)(b * Hkv + g)) * L + t];
        v = v * to_code;                               /* fp32, in [0, 127] */
        const float vh = f16_rne(v);                   /* the one rounding to FP16 */
        const float c1 = f16_rne(f16_rne(vh + 1536.0f) - 1536.0f);
        const float r = f16_rne(vh - c1);              /* exact */
        const float c2 = f16_rne(f16_rne(r * 254.0f + 1536.0f) - 1536.0f); /* r * 254 is exact in fp32: the fused form */
        p1[t] = (int8_t)c1;
        p2[t] = (int8_t)c2;
      }
    } else if (scale_mode == MSD_SCALE_PER_TOKEN) {
      const float apf = ap_num / 127.0f, bpf = apf / 254.0f;
      ap = apf;
      bp = bpf;
      for (int64_t t = 0; t < len; ++t) {
        const float pt = P[t] * v_scale[((int64_t)(b * Hkv + g)) * L + t];
        int c1 = 0, c2 = 0;
        if (apf > 0.0f) {
          c1 = clampi(rne_i(pt / apf), -128, 127);
          const float r = fmaf(-apf, (float)c1, pt);
          c2 = clampi(rne_i(r / bpf), -128, 127);
        }
        p1[t] = (int8_t)c1;
        p2[t] = (int8_t)c2;
      }
    } else {
      /* alpha_P = 1/127 is not an fp32 number: scale by the exact constants instead */
      ap = 1.0 / 127.0;
      bp = 1.0 / (127.0 * 254.0);
      for (int64_t t = 0; t < len; ++t) {
        const int c1 = clampi(rne_i(127.0f * P[t]), -128, 127);
        const float u = fmaf(127.0f, P[t], -(float)c1); /* r / alpha_P */
        p1[t] = (int8_t)c1;
        p2[t] = (int8_t)clampi(rne_i(u * 254.0f), -128, 127);
      }
    }
    for (int64_t t = 0; t < len; ++t) {
      if (tap_p) tap_p[(int64_t)bh * L + t] = P[t];
      if (tap_p1) tap_p1[(int64_t)bh * L + t] = p1[t];
      if (tap_p2) tap_p2[(int64_t)bh * L + t] = p2[t];
    }
    /* steps 10-13: O1, O2 integer GEMVs, merge, V scale, normalise */
    for (int c = 0; c < dv; ++c) {
      int64_t o1 = 0, o2 = 0;
      for (int64_t t = 0; t < len; ++t) {
        o1 += (int64_t)p1[t] * Vh[t * ldv + c];
        o2 += (int64_t)p2[t] * Vh[t * ldv + c];
      }
      double v = ap * (double)o1 + bp * (double)o2;
      if (scale_mode == MSD_SCALE_PER_CHANNEL) v *= (double)v_scale[g * dv + c];
      o[c] = (float)(v / ell);
    }
    free(qt); free(qf); free(q1); free(q2); free(S); free(P); free(p1); free(p2);
  }
}

void msd_oracle_attn_decode(const uint16_t* q_bf16, const int8_t* Kc, const int8_t* Vc,
                            const float* k_scale, const float* v_scale, int scale_mode, int B,
                            int Hq, int Hkv, int d, const int32_t* kv_len, int64_t L, float* out,
                            int8_t* tap_q1, int8_t* tap_q2, float* tap_alpha_q, int32_t* tap_s1,
                            int32_t* tap_s2, float* tap_p, int8_t* tap_p1, int8_t* tap_p2) {
  attn_decode_general(q_bf16, Kc, d, Vc, d, k_scale, v_scale, scale_mode, B, Hq, Hkv, d, d,
                      1.0 / sqrt((double)d), 0, kv_len, L, out, tap_q1, tap_q2, tap_alpha_q, tap_s1, tap_s2, tap_p,
                      tap_p1, tap_p2);
}

/* The same with the low-precision arithmetic described above attn_decode_general. */
void msd_oracle_attn_decode_lowprec(const uint16_t* q_bf16, const int8_t* Kc, const int8_t* Vc,
                                    const float* k_scale, const float* v_scale, int scale_mode, int B,
                                    int Hq, int Hkv, int d, const int32_t* kv_len, int64_t L, float* out,
                                    int8_t* tap_q1, int8_t* tap_q2, float* tap_alpha_q, int32_t* tap_s1,
                                    int32_t* tap_s2, float* tap_p, int8_t* tap_p1, int8_t* tap_p2) {
  attn_decode_general(q_bf16, Kc, d, Vc, d, k_scale, v_scale, scale_mode, B, Hq, Hkv, d, d,
                      1.0 / sqrt((double)d), 1, kv_len, L, out, tap_q1, tap_q2, tap_alpha_q, tap_s1, tap_s2, tap_p,
                      tap_p1, tap_p2);
}

/* ---------- the same for a latent KV cache (multi-head latent attention; Sec. 4.4, Sec. 7.3) ----
 * One cached row of ld >= dk INT8 values per token serves as key (its first dk channels: the latent
 * and the positional part) and as value (its first dv <= dk channels: the latent), shared by all Hq
 * query heads of a batch entry: Alg. 3 with Hkv = 1, K = C, V = C[:, :dv].  q [B][Hq][dk];
 * C [B][L][ld]; per-token scales scale[B][L] (the same scale for the key and the value reading of a
 * row) or per-channel scales scale[dk] (its first dv entries scale the values); out [B][Hq][dv];
 * the score scale sm_scale is the caller's (the absorbed form of such models does not use
 * 1/sqrt(dk)).  Taps as above with d = dk. */
void msd_oracle_mla_decode(const uint16_t* q_bf16, const int8_t* C, int64_t ld, const float* scale,
                           int scale_mode, int B, int Hq, int dk, int dv, double sm_scale,
                           const int32_t* kv_len, int64_t L, float* out, int8_t* tap_q1, int8_t* tap_q2,
                           float* tap_alpha_q, int32_t* tap_s1, int32_t* tap_s2) {
  attn_decode_general(q_bf16, C, ld, C, ld, scale, scale, scale_mode, B, Hq, 1, dk, dv, sm_scale, 0, kv_len, L, out,
                      tap_q1, tap_q2, tap_alpha_q, tap_s1, tap_s2, NULL, NULL, NULL);
}

/* fp64 truth: softmax(Q K_real^T / sqrt(d)) V_real with K_real, V_real the dequantised cache. */
static void truth_attn_general(const uint16_t* q_bf16, const int8_t* Kc, int64_t ldk, const int8_t* Vc,
                               int64_t ldv, const float* k_scale, const float* v_scale, int scale_mode,
                               int B, int Hq, int Hkv, int d, int dv, double sm_scale,
                               const int32_t* kv_len, int64_t L, double* out) {
  const int G = Hq / Hkv;
  const double inv_sqrt_d = sm_scale;
#pragma omp parallel for schedule(dynamic)
  for (int bh = 0; bh < B * Hq; ++bh) {
    const int b = bh / Hq, hq = bh % Hq, g = hq / G;
    int64_t len = kv_len ? kv_len[b] : L;
    if (len > L) len = L; /* entries past the cache are read as the cache length (the library clamps likewise) */
    const int64_t base = ((int64_t)(b * Hkv + g)) * L;
    double* o = out + (int64_t)bh * dv;
    for (int c = 0; c < dv; ++c) o[c] = 0.0;
    if (len <= 0) continue;
    double* S = (double*)malloc(sizeof(double) * (size_t)len);
    double smax = -INFINITY;
    for (int64_t t = 0; t < len; ++t) {
      double s = 0.0;
      for (int c = 0; c < d; ++c) {
        const double ks = scale_mode == MSD_SCALE_PER_TOKEN ? (double)k_scale[base + t]
                                                            : (double)k_scale[g * d + c];
        s += (double)bf16_to_f32(q_bf16[(int64_t)bh * d + c]) * ks * (double)Kc[(base + t) * ldk + c];
      }
      S[t] = s * inv_sqrt_d;
      if (S[t] > smax) smax = S[t];
    }
    double ell = 0.0;
    for (int64_t t = 0; t < len; ++t) {
      S[t] = exp(S[t] - smax);
      ell += S[t];
    }
    for (int64_t t = 0; t < len; ++t)
      for (int c = 0; c < dv; ++c) {
        const double vs = scale_mode == MSD_SCALE_PER_TOKEN ? (double)v_scale[base + t]
                                                            : (double)v_scale[g * dv + c];
        o[c] += S[t] * vs * (double)Vc[(base + t) * ldv + c];
      }
    for (int c = 0; c < dv; ++c) o[c] /= ell;
    free(S);
  }
}

void msd_oracle_truth_attn(const uint16_t* q_bf16, const int8_t* Kc, const int8_t* Vc,
                           const float* k_scale, const float* v_scale, int scale_mode, int B,
                           int Hq, int Hkv, int d, const int32_t* kv_len, int64_t L, double* out) {
  truth_attn_general(q_bf16, Kc, d, Vc, d, k_scale, v_scale, scale_mode, B, Hq, Hkv, d, d,
                     1.0 / sqrt((double)d), kv_len, L, out);
}

/* fp64 exact attention over the dequantised latent cache (see msd_oracle_mla_decode) */
void msd_oracle_truth_mla(const uint16_t* q_bf16, const int8_t* C, int64_t ld, const float* scale,
                          int scale_mode, int B, int Hq, int dk, int dv, double sm_scale,
                          const int32_t* kv_len, int64_t L, double* out) {
  truth_attn_general(q_bf16, C, ld, C, ld, scale, scale, scale_mode, B, Hq, 1, dk, dv, sm_scale, kv_len, L, out);
}

int msd_oracle_num_threads(void) {
  int n = 1;
#ifdef _OPENMP
#pragma omp parallel
  {
#pragma omp single
    n = omp_get_num_threads();
  }
#endif
  return n;
}
