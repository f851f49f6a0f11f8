/*
 * msd.h -- C ABI of the MI355X (gfx950) Multi-Scale Dequant library.
 *
 * Multi-Scale Dequant keeps quantised weights / KV caches in their storage format and
 * instead splits every BF16 activation vector into two low-precision components with
 * their own scales, x ~ alpha*x1 + beta*x2, so that both products run on native
 * low-precision matrix instructions and are merged by an fp32 epilogue (paper Sec. 1.2,
 * Sec. 3.1).
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller.  The library never
 *     allocates, frees, retains or synchronises: work is enqueued on `stream`
 *     (a hipStream_t passed as void*; NULL = the null stream) and the call returns.
 *   - Scratch memory comes from a caller-provided device `workspace` of at least
 *     msd_*_workspace_bytes(...) bytes, 256-byte aligned.  Its contents are undefined
 *     after the call.  Calls that share a workspace must be ordered on one stream.
 *   - BF16 tensors are raw 16-bit patterns.  Inputs must be finite.
 *   - GEMM shapes are (M, K, N): M activation rows (the paper's batch b), K the
 *     contraction length (the paper's n), N output channels (the paper's m).  Weights
 *     are stored [N][K] with K contiguous, so y[M][N] = X * W^T.
 *   - Return value: MSD_OK, or a negative error code; nothing is enqueued on error
 *     except for MSD_ERR_HIP, after which msd_last_hip_error() holds the hipError_t.
 *   - Results are deterministic run to run (no floating-point atomics).
 *   - The calls enqueue kernels only (plus device-to-device copies when observation points are
 *     requested), so they may be captured into a HIP graph.  The first call that reaches a kernel
 *     with a large LDS footprint sets that kernel's attribute (hipFuncSetAttribute): make one
 *     eager call of each shape class before capturing.
 */
#ifndef MSD_H_
#define MSD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  MSD_OK = 0,
  MSD_ERR_INVALID_ARG = -1, /* null / misaligned pointer, bad enum value */
  MSD_ERR_SHAPE = -2,       /* unsupported or inconsistent sizes */
  MSD_ERR_WORKSPACE = -3,   /* workspace null or too small */
  MSD_ERR_HIP = -4,         /* a HIP call failed; see msd_last_hip_error() */
  MSD_ERR_UNSUPPORTED = -5, /* valid request that this build has no kernel for */
  MSD_ERR_STATIC_SCRATCH = -6 /* msd_gemm_w8a16_static: the shape needs more scratch than the built-in buffer */
};

enum { MSD_INT8 = 0, MSD_MXFP4 = 1 };             /* decomposition format */
enum { MSD_F32 = 0, MSD_BF16 = 1 };               /* output dtype */
enum { MSD_PER_TOKEN = 0, MSD_PER_CHANNEL = 1 };  /* KV-cache scale granularity */
/* Parameterisations of the decomposition constants (paper Sec. 3.3).  MSD_VARIANT_MAIN is the
 * method as stated (what the entry points without a variant argument compute). */
enum {
  MSD_VARIANT_MAIN = 0,
  MSD_VARIANT_INT8_FRACTIONAL = 1, /* INT8: alpha = max|x| / 127.49, beta = alpha / 254.98 */
  MSD_VARIANT_MXFP4_V1 = 2,        /* MXFP4: alpha bound 1.75, beta = alpha / 8 (no clipping) */
  MSD_VARIANT_MXFP4_V2 = 3,        /* MXFP4: alpha bound 1.75, beta = alpha / 16 */
  MSD_VARIANT_MXFP4_E2M1 = 4,      /* MXFP4 ablation: both components on the MX FP4 element grid */
  MSD_VARIANT_ATTN_LOWPREC = 5     /* attention: integer S / O merge, FP16 decomposition of P (Sec. 4.4) */
};

/*
 * Optional observation points ("taps").  Any member may be NULL.  They exist so that the
 * integer intermediates of the method, which must be exact, can be compared from outside.
 *   GEMM W8A16 : q1,q2 int8 [M][K]; scale float alpha[M]; acc1,acc2 int32 [M][N]
 *   GEMM W4A16 : q1,q2 packed 4-bit codes [M][K/2]; scale uint8 E8M0 [M][K/32]; acc* unused
 *   attention  : q1,q2 int8 [B][Hq][d]; scale float alpha_Q [B][Hq]; acc1,acc2 int32 [B][Hq][L]
 *                (the two integer score rows S1, S2); p1,p2 int8 [B][Hq][L]: the two codes of the
 *                decomposed softmax numerator of every token, in units of that tile's alpha_P and
 *                alpha_P / 254 (msd_attn_decode_int8kv only, both or neither; other entry points ignore them)
 */
typedef struct msd_debug_taps {
  void* q1;
  void* q2;
  void* scale;
  int32_t* acc1;
  int32_t* acc2;
  void* p1;
  void* p2;
} msd_debug_taps;

/* hipError_t of the most recent failing HIP call made by this library on the calling thread. */
int msd_last_hip_error(void);
/* "major.minor" of this library; static storage. */
const char* msd_version(void);

/*
 * Two-pass activation decomposition of every row of x (paper Sec. 3.2, Eqs. for alpha, x1,
 * r, beta, x2; Sec. 3.2.1 / Alg. 2 for MXFP4).
 *   x_bf16 : [M][ldx] BF16, row m starts at x_bf16 + m*ldx; ldx >= K.
 *   fmt = MSD_INT8 : alpha = max|x_row| / 127, x1 = clamp(rne(x/alpha)), r = x - alpha*x1
 *       (fused multiply-add, one rounding), beta = alpha / 254, x2 = clamp(rne(r/beta));
 *       all in IEEE fp32 with correctly rounded division and round-half-to-even.
 *       q1,q2: int8 [M][K];  scale: float alpha[M] (beta is alpha/254).  K % 16 == 0.
 *       An all-zero row yields alpha = 0 and zero codes.
 *   fmt = MSD_MXFP4 : per block of 32 along K: alpha = 2^e with e the smallest integer such
 *       that max|x_block| <= 1.859375 * 2^e (clamped to [-123, 127]), q1 = nearest point of the
 *       uniform grid {k/4 : |k| <= 7} to x/alpha, r = x - alpha*q1 (exact), beta = alpha/16,
 *       q2 = nearest grid point to r/beta, saturating at +-7/4; ties to even k.
 *       q1,q2: uint8 [M][K/2], two 4-bit sign-magnitude codes per byte (bit 3 sign, bits 2..0 = k),
 *       low nibble = even k, -0 stored as +0;  scale: uint8 [M][K/32], E8M0 byte e+127 of alpha
 *       (beta's byte is that minus 4).  K % 32 == 0.  A zero block yields e = -123, zero codes.
 * Errors: INVALID_ARG (null pointer, bad fmt, x not 2-byte aligned), SHAPE (M,K < 0, ldx < K,
 * K not a multiple of 16 / 32).  M == 0 or K == 0 is a successful no-op.
 */
int msd_decompose(int fmt, const void* x_bf16, int64_t M, int64_t K, int64_t ldx, void* q1,
                  void* q2, void* scale, void* stream);

/*
 * MSD linear layer with INT8 weights (paper Alg. 1; Sec. 3.1 last equation; fused tiled
 * realisation of Sec. 3.9):  y = s_W (.) (alpha * (x1 W^T) + beta * (x2 W^T)).
 *   x_bf16  : [M][ldx] BF16 activations.
 *   W       : int8 [N][K], K contiguous, 16-byte aligned;  w_scale: float [N] per output channel.
 *   y       : [M][ldy] float (MSD_F32) or BF16 (MSD_BF16, round-to-nearest-even of the fp32 value).
 *   Both integer products are exact int32 accumulations (|K| <= 131072 guarantees no overflow);
 *   the merge and the weight scale are applied in fp32: y = s_W*(alpha*acc1 + beta*acc2).
 *   taps    : nullable, see msd_debug_taps.
 * Errors: INVALID_ARG, SHAPE (K % 16 != 0, K > 131072, ldx < K, ldy < N, negative sizes),
 * WORKSPACE.  M == 0 or N == 0 is a successful no-op; K == 0 writes zeros.
 */
int msd_gemm_w8a16(const void* x_bf16, int64_t M, int64_t K, int64_t ldx, const int8_t* W,
                   const float* w_scale, int64_t N, void* y, int out_dtype, int64_t ldy,
                   void* workspace, size_t workspace_bytes, const msd_debug_taps* taps,
                   void* stream);
size_t msd_gemm_w8a16_workspace_bytes(int64_t M, int64_t K, int64_t N);

/*
 * Pre-packed INT8 weights (optional, one time, offline; the weights stay INT8 and keep their size up to
 * padding).  The paper's kernels read the weights in the matrix unit's native tile format (Sec. 3.9: "resident
 * weight tile"); on gfx950 that is the lane order of the 16x16x64 integer matrix instruction's operand:
 *   packed[K/64][ceil(N/16)][1024]:  byte (g*16 + r)*16 + b of the kilobyte (ks, nb) = W[16*nb + r][64*ks + 16*g + b],
 *   zero for channels past N.
 * A load of one operand, or one fill instruction of an LDS tile, is then one contiguous kilobyte, which this
 * GPU serves at about three times the rate of 16 separate 64-byte row pieces.
 *   msd_packed_weights_w8_bytes(N, K) : size of the packed array (0 for empty shapes).
 *   msd_pack_weights_w8(W, N, K, packed, stream) : W int8 [N][K] (device) -> packed (device, 16-byte aligned).
 *       K must be a multiple of 64 (SHAPE error otherwise: such layers use msd_gemm_w8a16).
 *   msd_gemm_w8a16_packed(...) : msd_gemm_w8a16 with W_packed in place of W; every other argument, the
 *       workspace size (msd_gemm_w8a16_workspace_bytes), observation points, results (bit-identical integer
 *       partial products, the same fp32 epilogue) and errors as msd_gemm_w8a16, plus SHAPE for K % 64 != 0.
 */
size_t msd_packed_weights_w8_bytes(int64_t N, int64_t K);
int msd_pack_weights_w8(const int8_t* W, int64_t N, int64_t K, void* packed, void* stream);
int msd_gemm_w8a16_packed(const void* x_bf16, int64_t M, int64_t K, int64_t ldx, const void* W_packed,
                          const float* w_scale, int64_t N, void* y, int out_dtype, int64_t ldy,
                          void* workspace, size_t workspace_bytes, const msd_debug_taps* taps,
                          void* stream);

/*
 * msd_gemm_w8a16 for callers that cannot allocate device memory or carry a workspace (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc).  Same arguments, kernels and
 * results as msd_gemm_w8a16 without observation points; the activation codes and row scales live in a
 * buffer built into the library (device memory of msd_gemm_w8a16_static_scratch_bytes() = 2 MiB + 4 KiB
 * per GPU, held until the process ends) instead of a caller's workspace.  The call allocates and frees
 * nothing and synchronises nothing.
 *   Limit: msd_gemm_w8a16_workspace_bytes(M, K, N) - 256 must not exceed the buffer, i.e.
 *   2 * roundup(M, 128) * K + 4 * M (each term rounded up to 256) <= 2 MiB + 4 KiB: up to 128 rows at
 *   K <= 8192, 256 rows at K <= 4096.  Larger shapes return MSD_ERR_STATIC_SCRATCH and enqueue nothing.
 *   Every call on a GPU shares that GPU's buffer: calls must be ordered on one stream (or otherwise not
 *   overlap), concurrent calls on one GPU race.  The buffer keeps the previous call's contents; the
 *   kernels overwrite everything they later read, so nothing needs clearing.
 *   The first call on each device also resolves the buffer's device address (hipGetSymbolAddress) and,
 *   like msd_gemm_w8a16, may set a kernel attribute: make one eager call per shape class before capturing.
 * Other errors as msd_gemm_w8a16.
 */
int msd_gemm_w8a16_static(const void* x_bf16, int64_t M, int64_t K, int64_t ldx, const int8_t* W,
                          const float* w_scale, int64_t N, void* y, int out_dtype, int64_t ldy,
                          void* stream);
size_t msd_gemm_w8a16_static_scratch_bytes(void);

/*
 * MSD linear layer with MXFP4 weights (paper Sec. 3.2.1, Alg. 2, Sec. 3.4.1): the two
 * 4-bit activation components of every 32-block are multiplied against the MXFP4 weights
 * with block scales on both operands and summed in one fp32 accumulator.
 *   W_fp4  : uint8 [N][K/2], OCP E2M1 codes (bit 3 sign, bits 2..1 exponent, bit 0 mantissa),
 *            low nibble = even k, 16-byte aligned;  W_e8m0: uint8 [N][K/32], scale 2^(byte-127).
 *   y[m][n] = sum_blocks 2^(eW-127) * ( alpha_b * <q1_b, w_b> + beta_b * <q2_b, w_b> ), fp32.
 * Errors as msd_gemm_w8a16, with K % 32 != 0 a SHAPE error.
 */
int msd_gemm_w4a16(const void* x_bf16, int64_t M, int64_t K, int64_t ldx, const uint8_t* W_fp4,
                   const uint8_t* W_e8m0, int64_t N, void* y, int out_dtype, int64_t ldy,
                   void* workspace, size_t workspace_bytes, const msd_debug_taps* taps,
                   void* stream);
size_t msd_gemm_w4a16_workspace_bytes(int64_t M, int64_t K, int64_t N);

/*
 * Pre-packed MXFP4 weights (optional, one time, offline; same bits, regrouped -- the counterpart of
 * msd_pack_weights_w8 for the block-scaled matrix instructions, whose operand is 16 channels x 4 MX blocks):
 *   packed_fp4 [K/128][ceil(N/16)][1024]: byte ((g*16 + r)*16 + b) of the kilobyte (q, nb) =
 *       byte b of MX block 4q + g of channel 16*nb + r (W_fp4[16*nb + r][(4q + g)*16 + b]); zero past N.
 *   packed_e8m0, first part [K/512][ceil(N/16)][256]: byte (r*16 + i) of the record (s, nb) =
 *       W_e8m0[16*nb + r][16*s + i]; 0x7F past N.  Second part, at the next multiple of 256 bytes,
 *       [K/64][ceil(N/256)][512]: the same bytes in the order the many-row kernel stages them -- byte
 *       (r/128)*256 + b*128 + (r%32)*4 + (r/32)%4 of the record (t, nt) = W_e8m0[256*nt + r][2*t + b]; 0x7F past N
 *       -- so that no call has to rearrange them.
 * One operand load is then one contiguous kilobyte instead of 16 pieces of 64 bytes, and the 16 scale bytes of
 * 16 channels one 256-byte run.
 *   msd_packed_weights_w4_bytes / msd_packed_scales_w4_bytes (N, K): sizes of the two arrays (0 for empty shapes).
 *   msd_pack_weights_w4(W_fp4, W_e8m0, N, K, packed_fp4, packed_e8m0, stream): device arrays, the packed ones
 *       16-byte aligned.  K must be a multiple of 512 (SHAPE error otherwise: such layers use msd_gemm_w4a16).
 *   msd_gemm_w4a16_packed(...): msd_gemm_w4a16 on the packed arrays; other arguments, workspace size, observation
 *       points, results (bit-identical: same instructions on the same operands) and errors as msd_gemm_w4a16,
 *       plus SHAPE for K % 512 != 0 and UNSUPPORTED for row counts whose kernel does not read the packed layout.
 */
size_t msd_packed_weights_w4_bytes(int64_t N, int64_t K);
size_t msd_packed_scales_w4_bytes(int64_t N, int64_t K);
int msd_pack_weights_w4(const uint8_t* W_fp4, const uint8_t* W_e8m0, int64_t N, int64_t K, void* packed_fp4,
                        void* packed_e8m0, void* stream);
int msd_gemm_w4a16_packed(const void* x_bf16, int64_t M, int64_t K, int64_t ldx, const void* packed_fp4,
                          const void* packed_e8m0, int64_t N, void* y, int out_dtype, int64_t ldy,
                          void* workspace, size_t workspace_bytes, const msd_debug_taps* taps,
                          void* stream);

/*
 * The three entry points above with the decomposition constants of paper Sec. 3.3 selectable
 * ("fractional scaling" paragraph for INT8; the MXFP4 design-evolution table for MXFP4).
 * Everything else (arguments, layouts, workspace sizes, errors) is as for the entry point of the
 * same name without the suffix, which is the call with variant = MSD_VARIANT_MAIN.
 *   MSD_VARIANT_INT8_FRACTIONAL (msd_decompose with MSD_INT8, msd_gemm_w8a16): alpha =
 *       max|x_row| / 127.49f, beta = alpha / 254.98f (the two constants rounded to fp32), the merge
 *       uses the same beta; reconstruction bound max|x| / 65015 instead of / 64516.
 *   MSD_VARIANT_MXFP4_V1 (msd_decompose with MSD_MXFP4, msd_gemm_w4a16): e is the smallest
 *       integer with max|x_block| <= 1.75 * 2^e and beta = alpha / 8 (beta's E8M0 byte is alpha's
 *       minus 3); the residual never saturates.
 *   MSD_VARIANT_MXFP4_V2: bound 1.75 as v1, beta = alpha / 16 as the main variant.
 *   MSD_VARIANT_MXFP4_E2M1 (an ablation, not a parameterisation the paper prints): both components
 *       take values on the MX FP4 element grid {0, .5, 1, 1.5, 2, 3, 4, 6} (what a native FP4 x FP4
 *       product would consume) instead of the paper's uniform grid {k/4}: e is the smallest integer with
 *       max|x_block| <= 6 * 2^e, q1 = nearest grid value to x/alpha (ties to the even code),
 *       beta = alpha / 4 (byte minus 2), q2 = nearest grid value to r/beta (never saturates);
 *       |x - (alpha q1 + beta q2)| <= alpha / 8.  q1, q2 of msd_decompose and of the observation points
 *       are then OCP E2M1 nibbles (bit 3 sign, bits 2..1 exponent, bit 0 mantissa).
 * A variant that does not belong to the format of the call is an INVALID_ARG error.
 */
int msd_decompose_variant(int variant, int fmt, const void* x_bf16, int64_t M, int64_t K, int64_t ldx,
                          void* q1, void* q2, void* scale, void* stream);
int msd_gemm_w8a16_variant(int variant, const void* x_bf16, int64_t M, int64_t K, int64_t ldx,
                           const int8_t* W, const float* w_scale, int64_t N, void* y, int out_dtype,
                           int64_t ldy, void* workspace, size_t workspace_bytes,
                           const msd_debug_taps* taps, void* stream);
int msd_gemm_w4a16_variant(int variant, const void* x_bf16, int64_t M, int64_t K, int64_t ldx,
                           const uint8_t* W_fp4, const uint8_t* W_e8m0, int64_t N, void* y,
                           int out_dtype, int64_t ldy, void* workspace, size_t workspace_bytes,
                           const msd_debug_taps* taps, void* stream);

/*
 * Grouped MSD linear layer for mixture-of-experts models (paper Sec. 7.5: the decomposition works on
 * individual activation rows, so a grouped GEMM is msd_gemm_w8a16 per expert).  The T activation
 * rows are sorted by expert; expert e owns rows [expert_offsets[e], expert_offsets[e+1]) and
 * multiplies them with its own weights:
 *   y[t][:] = w_scale[e][:] (.) (alpha_t * (x1_t W[e]^T) + beta_t * (x2_t W[e]^T))   for t in expert e.
 *   expert_offsets : DEVICE int32 [E+1], non-decreasing, expert_offsets[0] = 0 and
 *                    expert_offsets[E] <= T (rows past it are left unwritten).  It is read by the
 *                    kernels; the host never looks at it, so no synchronisation is needed after routing.
 *   W : int8 [E][N][K];  w_scale : float [E][N];  x_bf16 : [T][ldx];  y : [T][ldy].
 *   workspace : msd_gemm_w8a16_workspace_bytes(T, K, N) bytes.
 * One decomposition launch over all rows and one GEMM launch over (channel tiles x experts);
 * experts without rows cost nothing but the launch of their workgroups.  Meant for decode, where
 * an expert sees a handful of rows (the kernel walks an expert's rows 16 at a time).
 * Errors as msd_gemm_w8a16; E > 65535 is a SHAPE error.
 */
int msd_moe_gemm_w8a16(const void* x_bf16, int64_t T, int64_t K, int64_t ldx,
                       const int32_t* expert_offsets, int E, const int8_t* W, const float* w_scale,
                       int64_t N, void* y, int out_dtype, int64_t ldy, void* workspace,
                       size_t workspace_bytes, void* stream);

/*
 * The same for MXFP4 weights: msd_gemm_w4a16 per expert.
 *   W_fp4 : uint8 [E][N][K/2];  W_e8m0 : uint8 [E][N][K/32];  other arguments as msd_moe_gemm_w8a16.
 *   workspace : msd_gemm_w4a16_workspace_bytes(T, K, N) bytes.
 * The kernel walks an expert's rows 8 at a time (both components of 8 rows fill one 16-row
 * matrix operand).
 */
int msd_moe_gemm_w4a16(const void* x_bf16, int64_t T, int64_t K, int64_t ldx,
                       const int32_t* expert_offsets, int E, const uint8_t* W_fp4,
                       const uint8_t* W_e8m0, int64_t N, void* y, int out_dtype, int64_t ldy,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * One decode step of attention over an INT8 KV cache without dequantising it (paper
 * Sec. 4.2, Alg. 3; tiling of Sec. 4.3): Q and the softmax numerator P are decomposed into
 * two INT8 components each, Q K^T and P V run as INT8 products, softmax is fp32 and online.
 *   q_bf16 : [B][Hq][d] BF16;  K, V: int8 [B][Hkv][L][d];  query head h reads KV head h/(Hq/Hkv).
 *   scale_mode MSD_PER_CHANNEL: k_scale, v_scale float [Hkv][d]; s_K is folded into Q before
 *       the decomposition, s_V multiplies the output (Alg. 3 as printed), alpha_P = 1/127.
 *       Both arrays are required (INVALID_ARG if NULL) even when L == 0.
 *   scale_mode MSD_PER_TOKEN : k_scale, v_scale float [B][Hkv][L]; s_K[t] multiplies score
 *       column t in the merge; P_t*s_V[t] is decomposed with alpha_P = (max s_V over the KV tile)/127.
 *   kv_len : nullable int32 [B], valid tokens per batch entry (<= L); NULL means L everywhere.
 *   out    : [B][Hq][d] float or BF16.  Entries with kv_len == 0 produce zeros.
 *   d must be 128 (64 and 256 are SHAPE errors in this version); Hq % Hkv == 0; Hq/Hkv <= 64.
 *   Up to 24 query heads per KV head share one pass over the KV cache (8 heads fill one 16-row
 *   matrix operand; two or three operands are held at once for 9..24 heads); larger groups are
 *   processed 16 heads per pass (also in the comparison kernel), each pass re-reading the split's
 *   KV range.
 */
int msd_attn_decode_int8kv(const void* q_bf16, const int8_t* K, const int8_t* V,
                           const float* k_scale, const float* v_scale, int scale_mode, int B,
                           int Hq, int Hkv, int d, const int32_t* kv_len, int64_t L, void* out,
                           int out_dtype, void* workspace, size_t workspace_bytes,
                           const msd_debug_taps* taps, void* stream);
size_t msd_attn_decode_int8kv_workspace_bytes(int B, int Hq, int Hkv, int d, int64_t L);

/*
 * msd_attn_decode_int8kv with the low-precision arithmetic the paper lists among its optimisation
 * opportunities (Sec. 4.4: the decomposition and the S / O merging in 16-bit arithmetic in place of fp32) for
 * variant = MSD_VARIANT_ATTN_LOWPREC; variant = MSD_VARIANT_MAIN is msd_attn_decode_int8kv itself.  What changes:
 *   - S = beta_Q * (254 S1 + S2) / sqrt(d) (times s_K[t]): the merge as one exact integer multiply-add, one
 *     conversion, one fp32 multiply (alpha_Q S1 + beta_Q S2 = beta_Q (254 S1 + S2) exactly);
 *   - P (times s_V[t]) / alpha_P, a number in [0, 127], is rounded once to FP16 (ties to even) and decomposed in
 *     FP16: P1 = rne(v), r = v - P1 (exact), P2 = rne(254 r); no clamp can fire.  Per element
 *     |v - (P1 + P2/254)| <= 2^-11 v + 1/508 in units of alpha_P, against 1/508 for the fp32 arithmetic;
 *   - O = beta_P * (254 O1 + O2) per tile, the same identity.
 * Q codes, alpha_Q and the integer score rows are unchanged (and bit-exact); outputs stay within 1e-3 of the
 * fp64 attention.  Arguments, workspace, observation points and errors as msd_attn_decode_int8kv; any other
 * variant is an INVALID_ARG error.
 */
int msd_attn_decode_int8kv_variant(int variant, const void* q_bf16, const int8_t* K, const int8_t* V,
                                   const float* k_scale, const float* v_scale, int scale_mode, int B,
                                   int Hq, int Hkv, int d, const int32_t* kv_len, int64_t L, void* out,
                                   int out_dtype, void* workspace, size_t workspace_bytes,
                                   const msd_debug_taps* taps, void* stream);

/*
 * One decode step of attention over an INT8 latent KV cache (multi-head latent attention; paper
 * Sec. 4.2 / Alg. 3 with the shapes of Sec. 4.4 and Sec. 7.3).  One cached row per token serves
 * every query head of a batch entry: its dk = 576 channels (512 latent + 64 positional) are the
 * key, its first dv = 512 channels the value.
 *   q_bf16 : [B][Hq][576] BF16 (the query in the cache's coordinates);  C : int8 [B][L][ld],
 *            ld >= 576 and a multiple of 16, 16-byte aligned.
 *   scale_mode MSD_PER_TOKEN : scale float [B][L], the scale of the whole cached row (it multiplies
 *            score column t and, folded into P, value row t);  MSD_PER_CHANNEL : scale float [576],
 *            folded into Q for the key reading, its first 512 entries multiply the output
 *            (required even when L == 0).
 *   sm_scale : the factor on the scores before the softmax (> 0; such models do not use 1/sqrt(576)).
 *   out    : [B][Hq][512] float or BF16.  kv_len, workspace, taps (q1, q2 int8 [B][Hq][576];
 *            scale = alpha_Q [B][Hq]; acc1, acc2 = the integer score rows [B][Hq][L]) as for
 *            msd_attn_decode_int8kv;  workspace of msd_mla_decode_int8kv_workspace_bytes(B, Hq, L).
 * Every 64-token tile of the cache is fetched once per workgroup and shared by up to 64 heads;
 * more heads are spread over further workgroups.  Launches: the main kernel and the merge of the
 * KV splits; above 32 heads also a query-decomposition kernel.
 * Errors: SHAPE (dk != 576, dv != 512, ld), INVALID_ARG, WORKSPACE.
 */
int msd_mla_decode_int8kv(const void* q_bf16, const int8_t* C, int64_t ld, const float* scale,
                          int scale_mode, int B, int Hq, int dk, int dv, float sm_scale,
                          const int32_t* kv_len, int64_t L, void* out, int out_dtype, void* workspace,
                          size_t workspace_bytes, const msd_debug_taps* taps, void* stream);
size_t msd_mla_decode_int8kv_workspace_bytes(int B, int Hq, int64_t L);

/*
 * Comparison kernel for msd_mla_decode_int8kv: the conventional path of paper Sec. 4.1 on the latent-cache
 * shape (every cached byte lifted from INT8 to BF16 before Q C^T and P C), as one fused kernel plus the merge
 * of the KV splits.  Same arguments, layouts, workspace size and errors; taps are ignored.  The bytes become
 * BF16 exactly, both products run on BF16 matrix instructions with fp32 accumulation, P (times the row's scale
 * in per-token mode) is rounded to BF16; a per-token scale multiplies the score column in fp32, a per-channel
 * scale is folded into Q (rounded to BF16) and its first 512 entries multiply the output.  A workgroup serves
 * 16 heads; further heads are further workgroups that read the same rows again.
 */
int msd_dequant_mla_decode_int8kv(const void* q_bf16, const int8_t* C, int64_t ld, const float* scale,
                                  int scale_mode, int B, int Hq, int dk, int dv, float sm_scale,
                                  const int32_t* kv_len, int64_t L, void* out, int out_dtype, void* workspace,
                                  size_t workspace_bytes, const msd_debug_taps* taps, void* stream);

/*
 * Comparison kernel for msd_attn_decode_int8kv: the conventional path of paper Sec. 4.1 (K and V
 * lifted from INT8 to BF16 before Q K^T and P V), as one fused kernel.  Same arguments, layouts,
 * workspace size (msd_attn_decode_int8kv_workspace_bytes) and errors; taps are ignored.  K and V
 * bytes become BF16 exactly, Q K^T and P V run on BF16 matrix instructions with fp32
 * accumulation, P (times s_V[t] in per-token mode) is rounded to BF16.  Per-token s_K[t]
 * multiplies the score column in fp32; per-channel s_K is folded into Q (rounded to BF16), s_V
 * multiplies the output.
 */
int msd_dequant_attn_decode_int8kv(const void* q_bf16, const int8_t* K, const int8_t* V,
                                   const float* k_scale, const float* v_scale, int scale_mode,
                                   int B, int Hq, int Hkv, int d, const int32_t* kv_len, int64_t L,
                                   void* out, int out_dtype, void* workspace, size_t workspace_bytes,
                                   const msd_debug_taps* taps, void* stream);

/*
 * Comparison kernels (the conventional path the paper argues against, Sec. 3.1 first
 * equation): weights are lifted to BF16 inside the kernel (bf16(s_W*W) for INT8, exact for
 * MXFP4) and multiplied on BF16 matrix instructions with fp32 accumulation.  Same
 * arguments as the MSD entry points; taps are ignored.  With M >= 256 and a workspace of
 * msd_dequant_gemm_workspace_bytes(M, K, N) bytes (16-byte aligned, room for a BF16 copy of
 * W) the literal two-step form runs: one pass writes bf16(W) to the workspace, then a tiled
 * BF16 GEMM built on the MSD prefill pipeline multiplies.  With a smaller or null workspace,
 * or fewer rows, the weights are lifted inside a single streaming kernel.
 */
size_t msd_dequant_gemm_workspace_bytes(int64_t M, int64_t K, int64_t N);
int msd_dequant_gemm_w8a16(const void* x_bf16, int64_t M, int64_t K, int64_t ldx, const int8_t* W,
                           const float* w_scale, int64_t N, void* y, int out_dtype, int64_t ldy,
                           void* workspace, size_t workspace_bytes, const msd_debug_taps* taps,
                           void* stream);
int msd_dequant_gemm_w4a16(const void* x_bf16, int64_t M, int64_t K, int64_t ldx,
                           const uint8_t* W_fp4, const uint8_t* W_e8m0, int64_t N, void* y,
                           int out_dtype, int64_t ldy, void* workspace, size_t workspace_bytes,
                           const msd_debug_taps* taps, void* stream);

/*
 * Measurement aid (not a step of the method; no paper passage).  Reads the row-major byte
 * matrix src [rows][row_bytes] (device) once, in the access pattern of the decode kernels'
 * weight stream, computes nothing and writes nothing.  bench.py times it next to the GEMM
 * calls: it is what the same weight bytes cost on this GPU with no arithmetic, launch
 * included.  row_bytes must be a positive multiple of 256, src 16-byte aligned; rows == 0
 * is a no-op.  Errors: MSD_ERR_INVALID_ARG, MSD_ERR_SHAPE, MSD_ERR_HIP.
 */
int msd_stream_read(const void* src, int64_t rows, int64_t row_bytes, void* stream);

/*
 * Measurement aid (not a step of the method; no paper passage).  Reads `bytes` bytes at src (device, 16-byte
 * aligned, bytes a multiple of 16) once as a linear array -- every wave instruction one contiguous kilobyte, the
 * pattern of the packed weight layouts, sixteen instructions in flight per lane -- and computes and writes nothing.
 * bench.py times it next to the calls on packed weights.  Errors: MSD_ERR_INVALID_ARG, MSD_ERR_SHAPE, MSD_ERR_HIP.
 */
int msd_stream_read_linear(const void* src, int64_t bytes, void* stream);

/*
 * Measurement aid (not a step of the method; no paper passage).  The rate of the matrix pipe on given operand
 * bits, with no data movement: 2048 waves (eight per CU) each read six operand fragments once from `operands`
 * (device, 64 KB, 16-byte aligned) and issue 8 * iters matrix instructions on them into eight accumulators --
 * fmt = MSD_INT8: v_mfma_i32_32x32x32_i8 (2 * 32768 operations each), fmt = MSD_MXFP4: the FP6 x FP4
 * block-scaled 32x32x64 instruction (2 * 65536 each), the instructions of the many-row GEMM kernels.  Timed by
 * bench.py with random and with constant buffers: the instruction rate in cycles is the same, the clock the chip
 * sustains under the load is not.  iters in [0, 2^22].  Errors: MSD_ERR_INVALID_ARG, MSD_ERR_SHAPE, MSD_ERR_HIP.
 */
int msd_probe_mfma_rate(int fmt, const void* operands, int iters, void* stream);

/*
 * Measurement aid (not a step of the method; no paper passage).  The rate at which the CUs can fill LDS, with no
 * arithmetic: 256 workgroups of eight waves; in each of `rounds` rounds a wave issues four asynchronous
 * 16-byte-per-lane loads into LDS (one contiguous kilobyte each: 32 KB per workgroup and round, 8 MB per round
 * over the grid) into a ring of four rounds, two rounds ahead, with a wait and a barrier per round -- the fill
 * instructions, depth and synchronisation of the tile GEMM kernels without their fragment reads and matrix
 * instructions.  src (device, 16-byte aligned, src_bytes a multiple of 1024): its first hot_bytes (a multiple of
 * 1024, at least 1024) are a window that every workgroup walks in the same order, wrapping (data that stays in
 * L2, like the activation codes); the remaining src_bytes - hot_bytes (at least 1024) are dealt to the workgroups
 * in disjoint ranges, wrapping at the end (data that streams from HBM when the range is large, like the weights).
 * hot_parts in [0, 4]: how many of a wave's four instructions per round read the window.  Nothing is written
 * outside LDS.  rounds in [0, 2^20].  Errors: MSD_ERR_INVALID_ARG, MSD_ERR_SHAPE, MSD_ERR_HIP.
 */
int msd_probe_lds_fill_rate(const void* src, int64_t src_bytes, int64_t hot_bytes, int hot_parts, int rounds,
                            void* stream);

/*
 * Measurement aid (not a step of the method; no paper passage).  Same arguments and the same
 * launches as msd_gemm_w8a16 on its many-row kernel (decomposition, then the 256x256-tile GEMM),
 * except that after the first K step the GEMM kernel stops fetching and keeps multiplying that
 * step's fragments: the same matrix-instruction sequence, tile schedule and epilogue on real
 * operand bits, with no tile fill, no barrier and no LDS traffic.  y receives meaningless
 * values.  Its time is what the matrix pipe alone allows for this shape and data on the GPU at
 * hand (the clock under matrix load depends on the operand bits).  Requires K % 64 == 0, fp32
 * output, workspace of msd_gemm_w8a16_workspace_bytes(M, K, N); taps are ignored.
 */
int msd_probe_mfma_w8a16(const void* x_bf16, int64_t M, int64_t K, int64_t ldx, const int8_t* W,
                         const float* w_scale, int64_t N, void* y, int out_dtype, int64_t ldy,
                         void* workspace, size_t workspace_bytes, const msd_debug_taps* taps,
                         void* stream);
/* The same aid for msd_gemm_w4a16's many-row kernel (M > 32, K % 64 == 0, workspace of
 * msd_gemm_w4a16_workspace_bytes(M, K, N)). */
int msd_probe_mfma_w4a16(const void* x_bf16, int64_t M, int64_t K, int64_t ldx, const uint8_t* W_fp4,
                         const uint8_t* W_e8m0, int64_t N, void* y, int out_dtype, int64_t ldy,
                         void* workspace, size_t workspace_bytes, const msd_debug_taps* taps,
                         void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MSD_H_ */
