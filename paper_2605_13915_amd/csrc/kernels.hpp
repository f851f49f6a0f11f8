// Internal launcher declarations of the gfx950 MSD library.
#pragma once
#include "msd_common.hpp"

namespace msd {

// ---- variants of the decomposition constants (paper Sec. 3.3)
// INT8: alpha = max|x| / num1, beta = alpha / num2; (127, 254) is the method as stated, (127.49, 254.98)
// the "fractional scaling" refinement with the bound M/65015.
struct Int8Range {
  float num1 = 127.0f, num2 = 254.0f;
};
// MXFP4: MxVariant (msd_common.hpp).

// ---- decomposition (decompose.hip)
// a_step != 0: write the blocked layout of GemmW8Args (stage depth a_bk) instead of row-major [M][ldq]
// frag_rt != 0: write the fragment-major layout (GemmW8Args::a_frag) with frag_rt fragments of 16 stacked rows
int launch_decompose_int8(const uint16_t* x, int64_t M, int64_t K, int64_t ldx, int8_t* q1,
                          int8_t* q2, int64_t ldq, float* alpha, int64_t a_step, int a_bk, Int8Range rg,
                          hipStream_t stream, int frag_rt = 0);
int launch_decompose_mxfp4(const uint16_t* x, int64_t M, int64_t K, int64_t ldx, uint8_t* abi_q1,
                           uint8_t* abi_q2, uint8_t* abi_e8m0, uint32_t* op_q1, uint32_t* op_q2,
                           uint8_t* op_e8m0, MxVariant mv, hipStream_t stream);

// ---- W8A16 dual INT8 GEMM + dual-scale epilogue (gemm_w8.hip)
struct GemmW8Args {
  const int8_t* q1;  // [M][ldq] first component codes
  const int8_t* q2;  // [M][ldq] residual component codes
  int64_t ldq;
  const float* alpha;  // [M]
  const int8_t* W;     // [N][K]
  const float* w_scale;
  void* y;
  int out_bf16;
  int64_t ldy;
  int32_t* acc1;  // nullable taps [M][N]
  int32_t* acc2;
  int64_t M, K, N;
  // single-launch decode (x == nullptr when the decomposition ran as its own kernel):
  const uint16_t* x;  // [M][ldx] BF16 activations
  int64_t ldx;
  int x_aligned;     // rows of x are 16-byte aligned
  int export_codes;  // also write q1/q2/alpha to the workspace (observation points)
  // blocked code layout for the asynchronous-fill kernels (a_step == 0: q1/q2 are row-major
  // [M][ldq]): q[K/a_bk stages][Mpad*a_bk/1024 blocks][1 KB], a block = 1024/a_bk rows of a_bk
  // bytes, the 16-byte chunks of a row stored at chunk ^ swizzle(row) (a_bk = 64: (row>>2)&3,
  // 128: (row>>1)&7), i.e. exactly the LDS image; a_step = bytes between stages, Mpad = M
  // rounded up to 128
  int64_t a_step;
  int a_bk;
  // fragment-major code layout for the register-operand kernels (a_frag = number of 16-row fragments RT, 0: off):
  // q1 holds both components, stacked row i = m or M + m; the 16 bytes of K step s, byte group g of stacked row
  // i sit at ((s * RT + i/16) * 64 + g * 16 + i%16) * 16, so that a wave's operand load is one contiguous
  // kilobyte (a load whose 64 lanes touch 16 different rows runs at a third of that rate)
  int a_frag;
  // packed weights (msd_pack_weights_w8): W points at Wp[K/64][Npad/16][1 KB], Npad = N rounded up to 16; the
  // kilobyte of K step ks and channel tile nb holds, at (g*16 + r)*16 + b, byte 64*ks + 16*g + b of channel
  // 16*nb + r (channels past N are zero) -- the lane order of the 16x16x64 matrix instruction's operand, so
  // a register-operand load and an LDS fill are one contiguous kilobyte each.  Requires K % 64 == 0.
  int w_packed;
  Int8Range rg;  // range constants of the decomposition and of beta in the epilogue
};
// stage depth of the blocked layout launch_gemm_w8 wants for this shape (0: row-major)
int gemm_w8_blocked_bk(int64_t M, int64_t K, int64_t N);
// number of 16-row fragments of the fragment-major layout launch_gemm_w8 wants for this shape (0: not used)
int gemm_w8_frag_rt(int64_t M, int64_t K, int64_t N);
// true when launch_gemm_w8 runs the decomposition itself (single launch)
bool gemm_w8_is_fused(int64_t M, int64_t K, int64_t N);
int launch_gemm_w8(const GemmW8Args& a, hipStream_t stream);
// grouped form (mixture of experts): a.q1/q2/alpha/y cover all T rows (row-major codes), a.W = [E][N][K],
// a.w_scale = [E][N]; expert e owns rows [offs[e], offs[e+1]) (device array of E + 1 entries); a.M is unused
int launch_gemm_w8_grouped(const GemmW8Args& a, const int32_t* offs, int E, hipStream_t stream);
// measurement aid: the prefill kernel's MFMA sequence, tile schedule and epilogue without fill,
// barriers and LDS traffic (output is meaningless); codes in the blocked layout or row-major
int launch_gemm_w8_mfma_probe(const GemmW8Args& a, hipStream_t stream);

// ---- W4A16 (gemm_w4.hip)
struct GemmW4Args {
  const uint32_t* q1;  // FP6 operand slots [M][K/32][8 dwords]
  const uint32_t* q2;
  const uint8_t* e8m0;  // alpha bytes [M][K/32]
  const uint8_t* W;     // [N][K/2]
  const uint8_t* We;    // [N][K/32]
  void* y;
  int out_bf16;
  int64_t ldy;
  int64_t M, K, N;
  // single-launch decode (x == nullptr when the decomposition ran as its own kernel):
  const uint16_t* x;
  int64_t ldx;
  int x_aligned;
  uint8_t* abi_q1;  // observation points in ABI format (nullable, all three or none)
  uint8_t* abi_q2;
  uint8_t* abi_e8m0;
  int scales_aligned;  // W_e8m0 is 16-byte aligned (16-byte scale loads allowed)
  int w_packed;        // W and We are the packed arrays of msd_pack_weights_w4 (needs K % 512 == 0)
  MxVariant mv;
};
bool gemm_w4_is_fused(int64_t M, int64_t K, int64_t N);
// grouped form (mixture of experts): a.q1/q2/e8m0/y cover all T rows, a.W = [E][N][K/2], a.We = [E][N][K/32];
// expert e owns rows [offs[e], offs[e+1]) (device array of E + 1 entries); a.M is unused
int launch_gemm_w4_grouped(const GemmW4Args& a, const int32_t* offs, int E, hipStream_t stream);
int launch_gemm_w4(const GemmW4Args& a, hipStream_t stream);
// one or two rows and many channels in one launch (a.x set; the kernel decomposes the rows once per workgroup)
bool gemm_w4_rows_applies(int64_t M, int64_t K, int64_t N, bool scales_aligned);
int launch_gemm_w4_rows(const GemmW4Args& a, hipStream_t stream);
// W [N][K/2], We [N][K/32] -> the packed arrays of msd_pack_weights_w4 (K % 512 == 0)
int launch_pack_weights_w4(const uint8_t* W, const uint8_t* We, int64_t N, int64_t K, uint8_t* Wp, uint8_t* Ep,
                           hipStream_t stream);

// ---- W4A16, many rows (gemm_w4_prefill.hip): own decomposition format, asynchronous LDS fill
struct GemmW4PrefillArgs {
  const uint8_t* qop;   // [M][K/64][96 B] FP6 operands of both components
  const uint8_t* sa_t;  // [K/64][Mpad][2] activation scale bytes (fetched with 32-bit offsets from this base)
  const uint8_t* sw_t;  // [K/64][Npad][2] weight scale bytes (likewise; workspace, or the packed array's second part)
  const uint8_t* W;     // [N][K/2], or the packed array of msd_pack_weights_w4
  int w_packed;
  void* y;
  int out_bf16;
  int64_t ldy;
  int64_t M, K, N, Mpad, Npad;
  MxVariant mv;
};
struct W4PrefillLayout {
  size_t qop, sa_t, sw_t, total, Mpad, Npad;
};
bool gemm_w4_prefill_applies(int64_t M, int64_t K, int64_t N);
W4PrefillLayout w4_prefill_layout(int64_t M, int64_t K, int64_t N);
// packed scale array of msd_pack_weights_w4: the decode-order records, then (256-byte aligned) the same bytes in the
// order of the many-row kernel's stages, [K/64][N rounded up to 256][2] with scale_slot inside a 256-column tile
size_t w4_packed_scales_decode_bytes(int64_t N, int64_t K);
size_t w4_packed_scales_bytes(int64_t N, int64_t K);
int launch_transpose_w_scales(const uint8_t* We, int64_t N, int64_t K, uint8_t* sw_t, hipStream_t stream);
// decomposition + scale transposition + GEMM; ws holds w4_prefill_layout(M, K, N).total bytes.
// probe: measurement aid -- the GEMM keeps multiplying the operands of its first K step (no fill,
// barriers or LDS traffic afterwards); y is then meaningless
int launch_gemm_w4_prefill(const uint16_t* x, int64_t ldx, const uint8_t* W, const uint8_t* We, void* y,
                           int out_bf16, int64_t ldy, int64_t M, int64_t K, int64_t N, uint8_t* ws,
                           MxVariant mv, hipStream_t stream, bool probe = false, int w_packed = 0);

// decomposition alone, in the K-step-major operand order described in gemm_w4_prefill.hip: qop holds
// (K/64) * (Mpad/32) * 3072 bytes, sa_t (K/64) * max(Mpad/256, 1) * 512 bytes; Mpad a multiple of 32
int launch_decompose_mxfp4_pair(const uint16_t* x, int64_t ldx, int64_t M, int64_t K, int64_t Mpad, uint8_t* qop,
                                uint8_t* sa_t, MxVariant mv, hipStream_t stream);

// ---- W4A16, 128 rows or fewer with the weight stream as the bound (gemm_w4_mid.hip)
struct W4MidLayout {
  size_t qop, sa_t, total, Mpad;  // Mpad: rows rounded up to 32, 64, 96 or 128
};
bool gemm_w4_mid_applies(int64_t M, int64_t K, int64_t N, bool scales_aligned);
W4MidLayout w4_mid_layout(int64_t M, int64_t K);
// decomposition (K-step-major operands of one, two or four 32-row groups) + GEMM; ws holds
// w4_mid_layout(M, K).total bytes
int launch_gemm_w4_mid(const uint16_t* x, int64_t ldx, const uint8_t* W, const uint8_t* We, void* y, int out_bf16,
                       int64_t ldy, int64_t M, int64_t K, int64_t N, uint8_t* ws, MxVariant mv, int w_packed,
                       hipStream_t stream);

// ---- attention (attn.hip)
struct AttnArgs {
  const uint16_t* q;
  const int8_t* K;
  const int8_t* V;
  const float* k_scale;
  const float* v_scale;
  int scale_mode;
  int B, Hq, Hkv, d;
  const int32_t* kv_len;
  int64_t L;
  void* out;
  int out_bf16;
  void* workspace;
  size_t workspace_bytes;
  const msd_debug_taps* taps;
  int lowprec;  // low-precision arithmetic of the softmax phase (Sec. 4.4, optimisation opportunities)
};
int launch_attn_decode(const AttnArgs& a, hipStream_t stream);
size_t attn_workspace_bytes(int B, int Hq, int Hkv, int d, int64_t L);
// comparison kernel (attn_dequant.hip): K and V lifted to BF16 in registers, BF16 matrix instructions;
// same arguments, split plan and workspace; taps are ignored
int launch_attn_dequant(const AttnArgs& a, hipStream_t stream);

// ---- attention over a latent KV cache (attn_mla.hip): keys = whole cached rows of 576 channels, values =
// their first 512, one row per token shared by all Hq heads of a batch entry
struct AttnMlaArgs {
  const uint16_t* q;   // [B][Hq][576]
  const int8_t* C;     // [B][L][ld]
  int64_t ld;
  const float* scale;  // per token [B][L] or per channel [576]
  int scale_mode;
  int B, Hq;
  float sm_scale;
  const int32_t* kv_len;
  int64_t L;
  void* out;           // [B][Hq][512]
  int out_bf16;
  void* workspace;
  const msd_debug_taps* taps;
};
int launch_attn_mla(const AttnMlaArgs& a, hipStream_t stream);
// the dequantise-then-BF16 comparison kernel on the same arguments (taps ignored)
int launch_attn_mla_dequant(const AttnMlaArgs& a, hipStream_t stream);
size_t attn_mla_workspace_bytes(int B, int Hq, int64_t L);

// ---- comparison kernels (dequant_gemm.hip)
// ws / ws_bytes: optional scratch for the BF16 copy of the weights (dequant_workspace_bytes);
// without it the fused single-kernel form runs whatever M is
int launch_dequant_gemm_w8(const uint16_t* x, int64_t M, int64_t K, int64_t ldx, const int8_t* W,
                           const float* w_scale, int64_t N, void* y, int out_bf16, int64_t ldy, void* ws,
                           size_t ws_bytes, hipStream_t stream);
int launch_dequant_gemm_w4(const uint16_t* x, int64_t M, int64_t K, int64_t ldx, const uint8_t* W,
                           const uint8_t* We, int64_t N, void* y, int out_bf16, int64_t ldy, void* ws,
                           size_t ws_bytes, hipStream_t stream);
size_t dequant_workspace_bytes(int64_t M, int64_t K, int64_t N);
// plain BF16 GEMM on the asynchronous-fill pipeline (gemm_w8.hip), used by the comparison path
int launch_bf16_gemm_tiled(const uint16_t* x, int64_t M, int64_t K, int64_t ldx, const uint16_t* Wb, int64_t N,
                           void* y, int out_bf16, int64_t ldy, hipStream_t stream);

// ---- one-time weight packing (gemm_w8.hip): W [N][K] -> the packed layout of GemmW8Args::w_packed
int launch_pack_weights_w8(const int8_t* W, int64_t N, int64_t K, int8_t* packed, hipStream_t stream);

// ---- measurement aid (stream_probe.hip)
int launch_stream_read(const void* src, int64_t rows, int64_t row_bytes, hipStream_t stream);
int launch_stream_read_linear(const void* src, int64_t bytes, hipStream_t stream);
// 1024 workgroups of two waves, each issuing 8 * iters matrix instructions on operands read once from a 64 KB buffer
int launch_mfma_rate(int fp4, const void* operands, int iters, hipStream_t stream);
// LDS fill rate alone (measurement aid): 256 workgroups x rounds x 32 KB of asynchronous LDS fills
int launch_lds_fill_rate(const void* src, int64_t src_bytes, int64_t hot_bytes, int hot_parts, int rounds,
                         hipStream_t stream);

}  // namespace msd
