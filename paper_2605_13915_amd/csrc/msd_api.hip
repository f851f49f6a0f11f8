// C-ABI entry points: argument validation, workspace carving, kernel dispatch.
#include <algorithm>
#include <mutex>

#include "kernels.hpp"

namespace msd {
thread_local int g_last_hip_error = 0;

// Built-in scratch of msd_gemm_w8a16_static: the activation codes and row scales that the other entry
// points keep in the caller's workspace.  One copy per GPU, held until the process ends.  In host code
// the array's name is only a handle for hipGetSymbolAddress; kernels and copies get the address that
// call returns on the device at hand.
constexpr size_t kStaticScratchBytes = (2u << 20) + 4096;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices] = {};

// device address of `scratch` on the current device, resolved once per device
static int static_scratch_ptr(void** out) {
  int dev = -1;
  MSD_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return MSD_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    MSD_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return MSD_ERR_UNSUPPORTED;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return MSD_OK;
}

__global__ void fill_u32_kernel(uint32_t* p, int64_t n, uint32_t v) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

static int fill_u32(uint32_t* p, int64_t n, uint32_t v, hipStream_t s) {
  if (n == 0) return MSD_OK;
  hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, s, p, n, v);
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

static bool aligned_to(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// workspace layout of msd_gemm_w8a16
struct W8Layout {
  size_t q1, q2, alpha, total;
};
static W8Layout w8_layout(int64_t M, int64_t K, int64_t N) {
  W8Layout l{};
  size_t off = 0;
  const size_t Mpad = align_up((size_t)M, 128);  // the blocked code layout holds whole 128-row tiles
  l.q1 = off; off = align_up(off + Mpad * K, 256);
  l.q2 = off; off = align_up(off + Mpad * K, 256);
  l.alpha = off; off = align_up(off + (size_t)M * sizeof(float), 256);
  l.total = off;
  return l;
}

// workspace layout of msd_gemm_w4a16
struct W4Layout {
  size_t q1, q2, e8m0, abi_q1, abi_q2, abi_e, total;
};
static W4Layout w4_layout(int64_t M, int64_t K, int64_t N) {
  W4Layout l{};
  const size_t KB = (size_t)K / 32;
  size_t off = 0;
  l.q1 = off; off = align_up(off + (size_t)M * KB * 32, 256);
  l.q2 = off; off = align_up(off + (size_t)M * KB * 32, 256);
  l.e8m0 = off; off = align_up(off + (size_t)M * KB, 256);
  l.total = off;
  // the many-row path keeps its own operand format; the workspace is sized for whichever is larger
  if (gemm_w4_prefill_applies(M, K, N)) l.total = std::max(l.total, w4_prefill_layout(M, K, N).total);
  if (gemm_w4_mid_applies(M, K, N, true)) l.total = std::max(l.total, w4_mid_layout(M, K).total);
  return l;
}
}  // namespace msd

using namespace msd;

// decomposition constants of a variant; false when the variant does not belong to the format
static bool int8_range_of(int variant, Int8Range& rg) {
  if (variant == MSD_VARIANT_MAIN) return true;
  if (variant != MSD_VARIANT_INT8_FRACTIONAL) return false;
  rg.num1 = 127.49f;
  rg.num2 = 254.98f;
  return true;
}
static bool mx_variant_of(int variant, MxVariant& mv) {
  if (variant == MSD_VARIANT_MAIN) return true;
  if (variant == MSD_VARIANT_MXFP4_E2M1) {  // both components on the MX FP4 element grid
    mv.hi_mant = 0x400000u;  // max|block| <= 6 alpha = 1.5 * 2^(e + 2)
    mv.ebias = 2;
    mv.shift = 2;
    mv.e2m1 = 1;
    return true;
  }
  if (variant != MSD_VARIANT_MXFP4_V1 && variant != MSD_VARIANT_MXFP4_V2) return false;
  mv.hi_mant = 0x600000u;  // 1.75
  mv.shift = variant == MSD_VARIANT_MXFP4_V1 ? 3 : 4;
  return true;
}

extern "C" {

int msd_last_hip_error(void) { return g_last_hip_error; }
const char* msd_version(void) { return "0.1"; }

int msd_decompose(int fmt, const void* x_bf16, int64_t M, int64_t K, int64_t ldx, void* q1, void* q2,
                  void* scale, void* stream) {
  return msd_decompose_variant(MSD_VARIANT_MAIN, fmt, x_bf16, M, K, ldx, q1, q2, scale, stream);
}

int msd_decompose_variant(int variant, int fmt, const void* x_bf16, int64_t M, int64_t K, int64_t ldx, void* q1,
                          void* q2, void* scale, void* stream) {
  if (fmt != MSD_INT8 && fmt != MSD_MXFP4) return MSD_ERR_INVALID_ARG;
  Int8Range rg;
  MxVariant mv;
  if (!(fmt == MSD_INT8 ? int8_range_of(variant, rg) : mx_variant_of(variant, mv))) return MSD_ERR_INVALID_ARG;
  if (M < 0 || K < 0 || ldx < K) return MSD_ERR_SHAPE;
  if (M == 0 || K == 0) return MSD_OK;
  if (!x_bf16 || !q1 || !q2 || !scale) return MSD_ERR_INVALID_ARG;
  if (!aligned_to(x_bf16, 2) || !aligned_to(q1, 16) || !aligned_to(q2, 16)) return MSD_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  if (fmt == MSD_INT8) {
    if (K % 16 != 0) return MSD_ERR_SHAPE;
    if (!aligned_to(scale, 4)) return MSD_ERR_INVALID_ARG;
    return launch_decompose_int8((const uint16_t*)x_bf16, M, K, ldx, (int8_t*)q1, (int8_t*)q2, K,
                                 (float*)scale, 0, 64, rg, s);
  }
  if (K % 32 != 0) return MSD_ERR_SHAPE;
  return launch_decompose_mxfp4((const uint16_t*)x_bf16, M, K, ldx, (uint8_t*)q1, (uint8_t*)q2,
                                (uint8_t*)scale, nullptr, nullptr, nullptr, mv, s);
}

size_t msd_gemm_w8a16_workspace_bytes(int64_t M, int64_t K, int64_t N) {
  if (M <= 0 || K < 0 || N <= 0) return 256;
  return w8_layout(M, K, N).total + 256;
}

int msd_gemm_w8a16(const void* x_bf16, int64_t M, int64_t K, int64_t ldx, const int8_t* W,
                   const float* w_scale, int64_t N, void* y, int out_dtype, int64_t ldy, void* workspace,
                   size_t workspace_bytes, const msd_debug_taps* taps, void* stream) {
  return msd_gemm_w8a16_variant(MSD_VARIANT_MAIN, x_bf16, M, K, ldx, W, w_scale, N, y, out_dtype, ldy, workspace,
                                workspace_bytes, taps, stream);
}

}  // extern "C"

// the W8A16 entry points: canonical [N][K] weights, or the packed layout of msd_pack_weights_w8
static int gemm_w4a16_impl(int variant, bool packed, const void* x_bf16, int64_t M, int64_t K, int64_t ldx,
                           const uint8_t* W_fp4, const uint8_t* W_e8m0, int64_t N, void* y, int out_dtype,
                           int64_t ldy, void* workspace, size_t workspace_bytes, const msd_debug_taps* taps,
                           void* stream);
static int gemm_w8a16_impl(int variant, bool packed, const void* x_bf16, int64_t M, int64_t K, int64_t ldx, const int8_t* W,
                           const float* w_scale, int64_t N, void* y, int out_dtype, int64_t ldy, void* workspace,
                           size_t workspace_bytes, const msd_debug_taps* taps, void* stream) {
  Int8Range rg;
  if (!int8_range_of(variant, rg)) return MSD_ERR_INVALID_ARG;
  if (out_dtype != MSD_F32 && out_dtype != MSD_BF16) return MSD_ERR_INVALID_ARG;
  if (M < 0 || K < 0 || N < 0 || ldx < K || ldy < N) return MSD_ERR_SHAPE;
  if (K % 16 != 0 || K > 131072) return MSD_ERR_SHAPE;
  if (packed && (K % 64 != 0 || K < 64)) return MSD_ERR_SHAPE;
  if (M == 0 || N == 0) return MSD_OK;
  if (!y || !w_scale || (K > 0 && (!x_bf16 || !W))) return MSD_ERR_INVALID_ARG;
  if (!aligned_to(W, 16) || !aligned_to(x_bf16, 2) || !aligned_to(w_scale, 4) ||
      !aligned_to(y, out_dtype == MSD_F32 ? 4 : 2))
    return MSD_ERR_INVALID_ARG;
  const W8Layout l = w8_layout(M, K, N);
  if (!workspace || !aligned_to(workspace, 256) || workspace_bytes < l.total) return MSD_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)workspace;
  GemmW8Args a{};
  a.w_packed = packed ? 1 : 0;
  a.q1 = (int8_t*)(ws + l.q1);
  a.q2 = (int8_t*)(ws + l.q2);
  a.ldq = K;
  a.alpha = (float*)(ws + l.alpha);
  a.W = W;
  a.w_scale = w_scale;
  a.y = y;
  a.out_bf16 = out_dtype == MSD_BF16;
  a.ldy = ldy;
  a.M = M; a.K = K; a.N = N;
  a.acc1 = taps ? taps->acc1 : nullptr;
  a.acc2 = taps ? taps->acc2 : nullptr;
  a.rg = rg;
  if (gemm_w8_is_fused(M, K, N)) {
    // one launch: the GEMM kernel decomposes the rows itself, under its own weight loads
    a.x = (const uint16_t*)x_bf16;
    a.ldx = ldx;
    a.x_aligned = (aligned_to(x_bf16, 16) && ldx % 8 == 0) ? 1 : 0;
    a.export_codes = (taps && (taps->q1 || taps->q2 || taps->scale)) ? 1 : 0;
  } else if (K > 0) {
    // codes in the layout the GEMM kernel of this shape reads; observation points want row-major
    const bool code_taps = taps && (taps->q1 || taps->q2);
    a.a_frag = code_taps ? 0 : gemm_w8_frag_rt(M, K, N);
    a.a_bk = (code_taps || a.a_frag) ? 0 : gemm_w8_blocked_bk(M, K, N);
    if (a.a_bk) a.a_step = (int64_t)align_up((size_t)M, 128) * a.a_bk;  // Mpad rows of a_bk bytes per stage
    int rc = launch_decompose_int8((const uint16_t*)x_bf16, M, K, ldx, (int8_t*)a.q1, (int8_t*)a.q2, K,
                                   (float*)a.alpha, a.a_step, a.a_bk ? a.a_bk : 64, rg, s, a.a_frag);
    if (rc) return rc;
  } else {
    int rc = fill_u32((uint32_t*)a.alpha, M, 0u, s);
    if (rc) return rc;
  }
  int rc = launch_gemm_w8(a, s);
  if (rc) return rc;
  if (taps && K > 0) {
    if (taps->q1) MSD_HIP_CHECK(hipMemcpyAsync(taps->q1, a.q1, (size_t)M * K, hipMemcpyDeviceToDevice, s));
    if (taps->q2) MSD_HIP_CHECK(hipMemcpyAsync(taps->q2, a.q2, (size_t)M * K, hipMemcpyDeviceToDevice, s));
    if (taps->scale)
      MSD_HIP_CHECK(hipMemcpyAsync(taps->scale, a.alpha, (size_t)M * 4, hipMemcpyDeviceToDevice, s));
  }
  return MSD_OK;
}

size_t msd_gemm_w8a16_static_scratch_bytes(void) { return kStaticScratchBytes; }

int msd_gemm_w8a16_static(const void* x_bf16, int64_t M, int64_t K, int64_t ldx, const int8_t* W,
                          const float* w_scale, int64_t N, void* y, int out_dtype, int64_t ldy, void* stream) {
  if (M < 0 || K < 0 || N < 0) return MSD_ERR_SHAPE;
  if (M > 0 && N > 0 && w8_layout(M, K, N).total > kStaticScratchBytes) return MSD_ERR_STATIC_SCRATCH;
  void* ptr = nullptr;
  const int rc = static_scratch_ptr(&ptr);
  if (rc) return rc;
  // Same kernels as msd_gemm_w8a16, with the built-in array in the workspace's place.  Nothing in it has
  // to start at zero: the decomposition launch writes every code and scale the GEMM launch looks at (rows
  // of a padded tile that it does not write only feed products that are never stored).
  return msd_gemm_w8a16_variant(MSD_VARIANT_MAIN, x_bf16, M, K, ldx, W, w_scale, N, y, out_dtype, ldy, ptr,
                                kStaticScratchBytes, nullptr, stream);
}

extern "C" {

int msd_gemm_w8a16_variant(int variant, const void* x_bf16, int64_t M, int64_t K, int64_t ldx, const int8_t* W,
                           const float* w_scale, int64_t N, void* y, int out_dtype, int64_t ldy, void* workspace,
                           size_t workspace_bytes, const msd_debug_taps* taps, void* stream) {
  return gemm_w8a16_impl(variant, false, x_bf16, M, K, ldx, W, w_scale, N, y, out_dtype, ldy, workspace, workspace_bytes,
                         taps, stream);
}

size_t msd_packed_weights_w8_bytes(int64_t N, int64_t K) {
  if (N <= 0 || K <= 0) return 0;
  return (size_t)((K + 63) / 64) * (size_t)((N + 15) / 16) * 1024;
}

int msd_pack_weights_w8(const int8_t* W, int64_t N, int64_t K, void* packed, void* stream) {
  if (N < 0 || K < 0 || K % 64 != 0 || K > 131072) return MSD_ERR_SHAPE;
  if (N == 0 || K == 0) return MSD_OK;
  if (!W || !packed || !aligned_to(W, 16) || !aligned_to(packed, 16)) return MSD_ERR_INVALID_ARG;
  return launch_pack_weights_w8(W, N, K, (int8_t*)packed, (hipStream_t)stream);
}

int msd_gemm_w8a16_packed(const void* x_bf16, int64_t M, int64_t K, int64_t ldx, const void* W_packed,
                          const float* w_scale, int64_t N, void* y, int out_dtype, int64_t ldy, void* workspace,
                          size_t workspace_bytes, const msd_debug_taps* taps, void* stream) {
  return gemm_w8a16_impl(MSD_VARIANT_MAIN, true, x_bf16, M, K, ldx, (const int8_t*)W_packed, w_scale, N, y, out_dtype,
                         ldy, workspace, workspace_bytes, taps, stream);
}

int msd_moe_gemm_w8a16(const void* x_bf16, int64_t T, int64_t K, int64_t ldx, const int32_t* expert_offsets, int E,
                       const int8_t* W, const float* w_scale, int64_t N, void* y, int out_dtype, int64_t ldy,
                       void* workspace, size_t workspace_bytes, void* stream) {
  if (out_dtype != MSD_F32 && out_dtype != MSD_BF16) return MSD_ERR_INVALID_ARG;
  if (T < 0 || K < 0 || N < 0 || E < 0 || ldx < K || ldy < N) return MSD_ERR_SHAPE;
  if (K % 16 != 0 || K > 131072 || E > 65535) return MSD_ERR_SHAPE;
  if (T == 0 || N == 0 || E == 0) return MSD_OK;
  if (!y || !w_scale || !expert_offsets || (K > 0 && (!x_bf16 || !W))) return MSD_ERR_INVALID_ARG;
  if (!aligned_to(W, 16) || !aligned_to(x_bf16, 2) || !aligned_to(w_scale, 4) || !aligned_to(expert_offsets, 4) ||
      !aligned_to(y, out_dtype == MSD_F32 ? 4 : 2))
    return MSD_ERR_INVALID_ARG;
  const W8Layout l = w8_layout(T, K, N);
  if (!workspace || !aligned_to(workspace, 256) || workspace_bytes < l.total) return MSD_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)workspace;
  GemmW8Args a{};
  a.q1 = (int8_t*)(ws + l.q1);
  a.q2 = (int8_t*)(ws + l.q2);
  a.ldq = K;
  a.alpha = (float*)(ws + l.alpha);
  a.W = W;
  a.w_scale = w_scale;
  a.y = y;
  a.out_bf16 = out_dtype == MSD_BF16;
  a.ldy = ldy;
  a.M = T; a.K = K; a.N = N;
  if (K > 0) {
    int rc = launch_decompose_int8((const uint16_t*)x_bf16, T, K, ldx, (int8_t*)a.q1, (int8_t*)a.q2, K,
                                   (float*)a.alpha, 0, 64, a.rg, s);
    if (rc) return rc;
  } else {
    int rc = fill_u32((uint32_t*)a.alpha, T, 0u, s);
    if (rc) return rc;
  }
  return launch_gemm_w8_grouped(a, expert_offsets, E, s);
}

size_t msd_gemm_w4a16_workspace_bytes(int64_t M, int64_t K, int64_t N) {
  if (M <= 0 || K <= 0 || N <= 0) return 256;
  return w4_layout(M, K, N).total + 256;
}

int msd_gemm_w4a16(const void* x_bf16, int64_t M, int64_t K, int64_t ldx, const uint8_t* W_fp4,
                   const uint8_t* W_e8m0, int64_t N, void* y, int out_dtype, int64_t ldy, void* workspace,
                   size_t workspace_bytes, const msd_debug_taps* taps, void* stream) {
  return msd_gemm_w4a16_variant(MSD_VARIANT_MAIN, x_bf16, M, K, ldx, W_fp4, W_e8m0, N, y, out_dtype, ldy,
                                workspace, workspace_bytes, taps, stream);
}

int msd_gemm_w4a16_variant(int variant, const void* x_bf16, int64_t M, int64_t K, int64_t ldx,
                           const uint8_t* W_fp4, const uint8_t* W_e8m0, int64_t N, void* y, int out_dtype,
                           int64_t ldy, void* workspace, size_t workspace_bytes, const msd_debug_taps* taps,
                           void* stream) {
  return gemm_w4a16_impl(variant, false, x_bf16, M, K, ldx, W_fp4, W_e8m0, N, y, out_dtype, ldy, workspace,
                         workspace_bytes, taps, stream);
}

size_t msd_packed_weights_w4_bytes(int64_t N, int64_t K) {
  if (N <= 0 || K <= 0) return 0;
  return (size_t)((K + 127) / 128) * (size_t)((N + 15) / 16) * 1024;
}

size_t msd_packed_scales_w4_bytes(int64_t N, int64_t K) {
  if (N <= 0 || K <= 0) return 0;
  return w4_packed_scales_bytes(N, K);
}

int msd_pack_weights_w4(const uint8_t* W_fp4, const uint8_t* W_e8m0, int64_t N, int64_t K, void* packed_fp4,
                        void* packed_e8m0, void* stream) {
  if (N < 0 || K < 0 || K % 512 != 0 || K > (1 << 20)) return MSD_ERR_SHAPE;
  if (N == 0 || K == 0) return MSD_OK;
  if (!W_fp4 || !W_e8m0 || !packed_fp4 || !packed_e8m0 || !aligned_to(W_fp4, 16) || !aligned_to(packed_fp4, 16) ||
      !aligned_to(packed_e8m0, 16))
    return MSD_ERR_INVALID_ARG;
  return launch_pack_weights_w4(W_fp4, W_e8m0, N, K, (uint8_t*)packed_fp4, (uint8_t*)packed_e8m0, (hipStream_t)stream);
}

int msd_gemm_w4a16_packed(const void* x_bf16, int64_t M, int64_t K, int64_t ldx, const void* packed_fp4,
                          const void* packed_e8m0, int64_t N, void* y, int out_dtype, int64_t ldy, void* workspace,
                          size_t workspace_bytes, const msd_debug_taps* taps, void* stream) {
  return gemm_w4a16_impl(MSD_VARIANT_MAIN, true, x_bf16, M, K, ldx, (const uint8_t*)packed_fp4,
                         (const uint8_t*)packed_e8m0, N, y, out_dtype, ldy, workspace, workspace_bytes, taps, stream);
}

}  // extern "C"

// the W4A16 entry points: canonical weights and scales, or the packed arrays of msd_pack_weights_w4
static int gemm_w4a16_impl(int variant, bool packed, const void* x_bf16, int64_t M, int64_t K, int64_t ldx,
                           const uint8_t* W_fp4, const uint8_t* W_e8m0, int64_t N, void* y, int out_dtype,
                           int64_t ldy, void* workspace, size_t workspace_bytes, const msd_debug_taps* taps,
                           void* stream) {
  MxVariant mv;
  if (!mx_variant_of(variant, mv)) return MSD_ERR_INVALID_ARG;
  if (out_dtype != MSD_F32 && out_dtype != MSD_BF16) return MSD_ERR_INVALID_ARG;
  if (M < 0 || K < 0 || N < 0 || ldx < K || ldy < N) return MSD_ERR_SHAPE;
  if (K % 32 != 0 || K > (1 << 20) || (packed && K % 512 != 0)) return MSD_ERR_SHAPE;
  if (M == 0 || N == 0) return MSD_OK;
  if (!y || (K > 0 && (!x_bf16 || !W_fp4 || !W_e8m0))) return MSD_ERR_INVALID_ARG;
  if (!aligned_to(W_fp4, 16) ||  !aligned_to(x_bf16, 2) || (packed && !aligned_to(W_e8m0, 16)) ||
      !aligned_to(y, out_dtype == MSD_F32 ? 4 : 2))
    return MSD_ERR_INVALID_ARG;
  const W4Layout l = w4_layout(M, K, N);
  if (!workspace || !aligned_to(workspace, 256) || workspace_bytes < l.total) return MSD_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)workspace;
  GemmW4Args a{};
  a.q1 = (uint32_t*)(ws + l.q1);
  a.q2 = (uint32_t*)(ws + l.q2);
  a.e8m0 = (uint8_t*)(ws + l.e8m0);
  a.W = W_fp4;
  a.We = W_e8m0;
  a.scales_aligned = aligned_to(W_e8m0, 16) ? 1 : 0;
  a.w_packed = packed ? 1 : 0;
  a.y = y;
  a.out_bf16 = out_dtype == MSD_BF16;
  a.ldy = ldy;
  a.M = M; a.K = K; a.N = N;
  a.mv = mv;
  if (K > 0) {
    uint8_t* t1 = taps ? (uint8_t*)taps->q1 : nullptr;
    uint8_t* t2 = taps ? (uint8_t*)taps->q2 : nullptr;
    uint8_t* te = taps ? (uint8_t*)taps->scale : nullptr;
    if (!(t1 && t2 && te)) t1 = t2 = te = nullptr;  // the ABI-format taps come as a set
    if (t1 && (!aligned_to(t1, 16) || !aligned_to(t2, 16))) return MSD_ERR_INVALID_ARG;
    // packed weights: every kernel of the product path reads them; observation points above 16 rows come from a
    // kernel that reads the canonical layout only, and so does the fallback for workspaces past 2 GiB
    if (packed && ((t1 && M > 16) || (M > 128 && w4_prefill_layout(M, K, N).total >= ((size_t)1 << 31))))
      return MSD_ERR_UNSUPPORTED;
    if (!t1 && gemm_w4_mid_applies(M, K, N, a.scales_aligned != 0)) {
      // 3..128 rows, no observation points: activation operands K-step-major, weights and operands
      // staged through LDS per 128 channels (the weight stream is the bound)
      return launch_gemm_w4_mid((const uint16_t*)x_bf16, ldx, W_fp4, W_e8m0, y, a.out_bf16, ldy, M, K, N,
                                (uint8_t*)ws, mv, a.w_packed, s);
    }
    if (!t1 && gemm_w4_prefill_applies(M, K, N) && w4_prefill_layout(M, K, N).total < ((size_t)1 << 31)) {
      // many rows, no observation points: decomposition in the GEMM's own operand order,
      // weight scales transposed once, GEMM on the asynchronous-fill pipeline
      return launch_gemm_w4_prefill((const uint16_t*)x_bf16, ldx, W_fp4, W_e8m0, y, a.out_bf16, ldy, M, K, N,
                                    (uint8_t*)ws, mv, s, false, a.w_packed);
    }
    if (!t1 && gemm_w4_rows_applies(M, K, N, a.scales_aligned != 0)) {
      // one or two rows, many channels: one launch, the rows decomposed once per workgroup
      a.x = (const uint16_t*)x_bf16;
      a.ldx = ldx;
      a.x_aligned = (aligned_to(x_bf16, 16) && ldx % 8 == 0) ? 1 : 0;
      return launch_gemm_w4_rows(a, s);
    }
    if (gemm_w4_is_fused(M, K, N) && !packed) {
      // one launch: the GEMM kernel decomposes the blocks of its own K range itself.  (On packed weights the
      // two-launch form measured faster, 29.6 vs 35.5 us at 1 x 8192 x 28672: the weight stream then runs at the
      // rate of a bare read and every workgroup's decomposition prologue shows.)
      a.x = (const uint16_t*)x_bf16;
      a.ldx = ldx;
      a.x_aligned = (aligned_to(x_bf16, 16) && ldx % 8 == 0) ? 1 : 0;
      a.abi_q1 = t1; a.abi_q2 = t2; a.abi_e8m0 = te;
    } else {
      int rc = launch_decompose_mxfp4((const uint16_t*)x_bf16, M, K, ldx, t1, t2, te, (uint32_t*)a.q1,
                                      (uint32_t*)a.q2, (uint8_t*)a.e8m0, mv, s);
      if (rc) return rc;
    }
  }
  return launch_gemm_w4(a, s);
}

extern "C" {

int msd_moe_gemm_w4a16(const void* x_bf16, int64_t T, int64_t K, int64_t ldx, const int32_t* expert_offsets, int E,
                       const uint8_t* W_fp4, const uint8_t* W_e8m0, int64_t N, void* y, int out_dtype, int64_t ldy,
                       void* workspace, size_t workspace_bytes, void* stream) {
  if (out_dtype != MSD_F32 && out_dtype != MSD_BF16) return MSD_ERR_INVALID_ARG;
  if (T < 0 || K < 0 || N < 0 || E < 0 || ldx < K || ldy < N) return MSD_ERR_SHAPE;
  if (K % 32 != 0 || K > (1 << 20) || E > 65535) return MSD_ERR_SHAPE;
  if (T == 0 || N == 0 || E == 0) return MSD_OK;
  if (!y || !expert_offsets || (K > 0 && (!x_bf16 || !W_fp4 || !W_e8m0))) return MSD_ERR_INVALID_ARG;
  if (!aligned_to(W_fp4, 16) || !aligned_to(x_bf16, 2) || !aligned_to(expert_offsets, 4) ||
      !aligned_to(y, out_dtype == MSD_F32 ? 4 : 2))
    return MSD_ERR_INVALID_ARG;
  const W4Layout l = w4_layout(T, K, N);
  if (!workspace || !aligned_to(workspace, 256) || workspace_bytes < l.total) return MSD_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)workspace;
  GemmW4Args a{};
  a.q1 = (uint32_t*)(ws + l.q1);
  a.q2 = (uint32_t*)(ws + l.q2);
  a.e8m0 = (uint8_t*)(ws + l.e8m0);
  a.W = W_fp4;
  a.We = W_e8m0;
  // every expert's scale rows must be 16-byte aligned for the 16-byte scale loads
  a.scales_aligned = (aligned_to(W_e8m0, 16) && (N * (K / 32)) % 16 == 0) ? 1 : 0;
  a.y = y;
  a.out_bf16 = out_dtype == MSD_BF16;
  a.ldy = ldy;
  a.M = T; a.K = K; a.N = N;
  if (K > 0) {
    int rc = launch_decompose_mxfp4((const uint16_t*)x_bf16, T, K, ldx, nullptr, nullptr, nullptr, (uint32_t*)a.q1,
                                    (uint32_t*)a.q2, (uint8_t*)a.e8m0, a.mv, s);
    if (rc) return rc;
  }
  return launch_gemm_w4_grouped(a, expert_offsets, E, s);
}

size_t msd_attn_decode_int8kv_workspace_bytes(int B, int Hq, int Hkv, int d, int64_t L) {
  if (B <= 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || L < 0) return 256;
  return attn_workspace_bytes(B, Hq, Hkv, d, L) + 256;
}

}  // extern "C"

static int attn_entry(bool dequant, bool lowprec, const void* q_bf16, const int8_t* K, const int8_t* V, const float* k_scale,
                           const float* v_scale, int scale_mode, int B, int Hq, int Hkv, int d,
                           const int32_t* kv_len, int64_t L, void* out, int out_dtype, void* workspace,
                           size_t workspace_bytes, const msd_debug_taps* taps, void* stream) {
  if (out_dtype != MSD_F32 && out_dtype != MSD_BF16) return MSD_ERR_INVALID_ARG;
  if (scale_mode != MSD_PER_TOKEN && scale_mode != MSD_PER_CHANNEL) return MSD_ERR_INVALID_ARG;
  if (B < 0 || Hq <= 0 || Hkv <= 0 || L < 0) return MSD_ERR_SHAPE;
  if (d != 128 || Hq % Hkv != 0 || Hq / Hkv > 64 || L > (1 << 24)) return MSD_ERR_SHAPE;
  if (B == 0) return MSD_OK;
  if (!q_bf16 || !out || (L > 0 && (!K || !V || !k_scale || !v_scale))) return MSD_ERR_INVALID_ARG;
  if (scale_mode == MSD_PER_CHANNEL && (!k_scale || !v_scale)) return MSD_ERR_INVALID_ARG;  // read even when L == 0
  if (!aligned_to(K, 16) || !aligned_to(V, 16) || !aligned_to(q_bf16, 16) || !aligned_to(out, 16))
    return MSD_ERR_INVALID_ARG;
  const size_t need = attn_workspace_bytes(B, Hq, Hkv, d, L);
  if (!workspace || !aligned_to(workspace, 256) || workspace_bytes < need) return MSD_ERR_WORKSPACE;
  AttnArgs a{};
  a.q = (const uint16_t*)q_bf16;
  a.K = K; a.V = V;
  a.k_scale = k_scale; a.v_scale = v_scale;
  a.scale_mode = scale_mode;
  a.B = B; a.Hq = Hq; a.Hkv = Hkv; a.d = d;
  a.kv_len = kv_len;
  a.L = L;
  a.out = out;
  a.out_bf16 = out_dtype == MSD_BF16;
  a.workspace = workspace;
  a.workspace_bytes = workspace_bytes;
  a.taps = dequant ? nullptr : taps;
  a.lowprec = lowprec ? 1 : 0;
  return dequant ? launch_attn_dequant(a, (hipStream_t)stream) : launch_attn_decode(a, (hipStream_t)stream);
}

extern "C" {

int msd_attn_decode_int8kv(const void* q_bf16, const int8_t* K, const int8_t* V, const float* k_scale,
                           const float* v_scale, int scale_mode, int B, int Hq, int Hkv, int d,
                           const int32_t* kv_len, int64_t L, void* out, int out_dtype, void* workspace,
                           size_t workspace_bytes, const msd_debug_taps* taps, void* stream) {
  return attn_entry(false, false, q_bf16, K, V, k_scale, v_scale, scale_mode, B, Hq, Hkv, d, kv_len, L, out, out_dtype,
                    workspace, workspace_bytes, taps, stream);
}

int msd_attn_decode_int8kv_variant(int variant, const void* q_bf16, const int8_t* K, const int8_t* V,
                                   const float* k_scale, const float* v_scale, int scale_mode, int B, int Hq, int Hkv,
                                   int d, const int32_t* kv_len, int64_t L, void* out, int out_dtype, void* workspace,
                                   size_t workspace_bytes, const msd_debug_taps* taps, void* stream) {
  if (variant != MSD_VARIANT_MAIN && variant != MSD_VARIANT_ATTN_LOWPREC) return MSD_ERR_INVALID_ARG;
  return attn_entry(false, variant == MSD_VARIANT_ATTN_LOWPREC, q_bf16, K, V, k_scale, v_scale, scale_mode, B, Hq, Hkv,
                    d, kv_len, L, out, out_dtype, workspace, workspace_bytes, taps, stream);
}

int msd_dequant_attn_decode_int8kv(const void* q_bf16, const int8_t* K, const int8_t* V, const float* k_scale,
                                   const float* v_scale, int scale_mode, int B, int Hq, int Hkv, int d,
                                   const int32_t* kv_len, int64_t L, void* out, int out_dtype, void* workspace,
                                   size_t workspace_bytes, const msd_debug_taps* taps, void* stream) {
  return attn_entry(true, false, q_bf16, K, V, k_scale, v_scale, scale_mode, B, Hq, Hkv, d, kv_len, L, out, out_dtype,
                    workspace, workspace_bytes, taps, stream);
}

size_t msd_mla_decode_int8kv_workspace_bytes(int B, int Hq, int64_t L) {
  if (B <= 0 || Hq <= 0 || L < 0) return 256;
  return attn_mla_workspace_bytes(B, Hq, L) + 256;
}

static int mla_decode_impl(bool dequant, const void* q_bf16, const int8_t* C, int64_t ld, const float* scale,
                           int scale_mode, int B, int Hq, int dk, int dv, float sm_scale, const int32_t* kv_len,
                           int64_t L, void* out, int out_dtype, void* workspace, size_t workspace_bytes,
                           const msd_debug_taps* taps, void* stream) {
  if (out_dtype != MSD_F32 && out_dtype != MSD_BF16) return MSD_ERR_INVALID_ARG;
  if (scale_mode != MSD_PER_TOKEN && scale_mode != MSD_PER_CHANNEL) return MSD_ERR_INVALID_ARG;
  if (B < 0 || Hq <= 0 || L < 0) return MSD_ERR_SHAPE;
  if (dk != 576 || dv != 512 || ld < dk || ld % 16 != 0 || L > (1 << 24)) return MSD_ERR_SHAPE;
  if (!(sm_scale > 0.f)) return MSD_ERR_INVALID_ARG;
  if (B == 0) return MSD_OK;
  if (!q_bf16 || !out || (L > 0 && (!C || !scale))) return MSD_ERR_INVALID_ARG;
  if (scale_mode == MSD_PER_CHANNEL && !scale) return MSD_ERR_INVALID_ARG;  // read even when L == 0
  if (!aligned_to(C, 16) || !aligned_to(q_bf16, 2) || !aligned_to(scale, 4) || !aligned_to(out, out_dtype == MSD_F32 ? 4 : 2))
    return MSD_ERR_INVALID_ARG;
  const size_t need = attn_mla_workspace_bytes(B, Hq, L);
  if (!workspace || !aligned_to(workspace, 256) || workspace_bytes < need) return MSD_ERR_WORKSPACE;
  AttnMlaArgs a{};
  a.q = (const uint16_t*)q_bf16;
  a.C = C;
  a.ld = ld;
  a.scale = scale;
  a.scale_mode = scale_mode;
  a.B = B; a.Hq = Hq;
  a.sm_scale = sm_scale;
  a.kv_len = kv_len;
  a.L = L;
  a.out = out;
  a.out_bf16 = out_dtype == MSD_BF16;
  a.workspace = workspace;
  a.taps = taps;
  return dequant ? launch_attn_mla_dequant(a, (hipStream_t)stream) : launch_attn_mla(a, (hipStream_t)stream);
}

int msd_mla_decode_int8kv(const void* q_bf16, const int8_t* C, int64_t ld, const float* scale, int scale_mode, int B,
                          int Hq, int dk, int dv, float sm_scale, const int32_t* kv_len, int64_t L, void* out,
                          int out_dtype, void* workspace, size_t workspace_bytes, const msd_debug_taps* taps,
                          void* stream) {
  return mla_decode_impl(false, q_bf16, C, ld, scale, scale_mode, B, Hq, dk, dv, sm_scale, kv_len, L, out, out_dtype,
                         workspace, workspace_bytes, taps, stream);
}

int msd_dequant_mla_decode_int8kv(const void* q_bf16, const int8_t* C, int64_t ld, const float* scale,
                                  int scale_mode, int B, int Hq, int dk, int dv, float sm_scale,
                                  const int32_t* kv_len, int64_t L, void* out, int out_dtype, void* workspace,
                                  size_t workspace_bytes, const msd_debug_taps* /*taps*/, void* stream) {
  return mla_decode_impl(true, q_bf16, C, ld, scale, scale_mode, B, Hq, dk, dv, sm_scale, kv_len, L, out, out_dtype,
                         workspace, workspace_bytes, nullptr, stream);
}

int msd_dequant_gemm_w8a16(const void* x_bf16, int64_t M, int64_t K, int64_t ldx, const int8_t* W,
                           const float* w_scale, int64_t N, void* y, int out_dtype, int64_t ldy,
                           void* workspace, size_t workspace_bytes, const msd_debug_taps* /*taps*/,
                           void* stream) {
  if (out_dtype != MSD_F32 && out_dtype != MSD_BF16) return MSD_ERR_INVALID_ARG;
  if (M < 0 || K < 0 || N < 0 || ldx < K || ldy < N) return MSD_ERR_SHAPE;
  if (K % 16 != 0) return MSD_ERR_SHAPE;
  if (M == 0 || N == 0) return MSD_OK;
  if (!y || !w_scale || (K > 0 && (!x_bf16 || !W))) return MSD_ERR_INVALID_ARG;
  if (!aligned_to(W, 16) || !aligned_to(x_bf16, 16) || ldx % 8 != 0) return MSD_ERR_INVALID_ARG;
  return launch_dequant_gemm_w8((const uint16_t*)x_bf16, M, K, ldx, W, w_scale, N, y,
                                out_dtype == MSD_BF16, ldy, workspace, workspace_bytes, (hipStream_t)stream);
}

int msd_dequant_gemm_w4a16(const void* x_bf16, int64_t M, int64_t K, int64_t ldx, const uint8_t* W_fp4,
                           const uint8_t* W_e8m0, int64_t N, void* y, int out_dtype, int64_t ldy,
                           void* workspace, size_t workspace_bytes, const msd_debug_taps* /*taps*/,
                           void* stream) {
  if (out_dtype != MSD_F32 && out_dtype != MSD_BF16) return MSD_ERR_INVALID_ARG;
  if (M < 0 || K < 0 || N < 0 || ldx < K || ldy < N) return MSD_ERR_SHAPE;
  if (K % 32 != 0) return MSD_ERR_SHAPE;
  if (M == 0 || N == 0) return MSD_OK;
  if (!y || (K > 0 && (!x_bf16 || !W_fp4 || !W_e8m0))) return MSD_ERR_INVALID_ARG;
  if (!aligned_to(W_fp4, 16) || !aligned_to(x_bf16, 16) || ldx % 8 != 0) return MSD_ERR_INVALID_ARG;
  return launch_dequant_gemm_w4((const uint16_t*)x_bf16, M, K, ldx, W_fp4, W_e8m0, N, y,
                                out_dtype == MSD_BF16, ldy, workspace, workspace_bytes, (hipStream_t)stream);
}

int msd_probe_mfma_w8a16(const void* x_bf16, int64_t M, int64_t K, int64_t ldx, const int8_t* W,
                         const float* w_scale, int64_t N, void* y, int out_dtype, int64_t ldy, void* workspace,
                         size_t workspace_bytes, const msd_debug_taps* /*taps*/, void* stream) {
  if (out_dtype != MSD_F32) return MSD_ERR_INVALID_ARG;
  if (M <= 0 || N <= 0 || K < 64 || K % 64 != 0 || K > 131072 || ldx < K || ldy < N) return MSD_ERR_SHAPE;
  if (!y || !w_scale || !x_bf16 || !W) return MSD_ERR_INVALID_ARG;
  if (!aligned_to(W, 16) || !aligned_to(x_bf16, 2) || !aligned_to(w_scale, 4) || !aligned_to(y, 4))
    return MSD_ERR_INVALID_ARG;
  const W8Layout l = w8_layout(M, K, N);
  if (!workspace || !aligned_to(workspace, 256) || workspace_bytes < l.total) return MSD_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)workspace;
  GemmW8Args a{};
  a.q1 = (int8_t*)(ws + l.q1);
  a.q2 = (int8_t*)(ws + l.q2);
  a.ldq = K;
  a.alpha = (float*)(ws + l.alpha);
  a.W = W;
  a.w_scale = w_scale;
  a.y = y;
  a.ldy = ldy;
  a.M = M; a.K = K; a.N = N;
  a.a_bk = 64;
  a.a_step = (int64_t)align_up((size_t)M, 128) * 64;
  int rc = launch_decompose_int8((const uint16_t*)x_bf16, M, K, ldx, (int8_t*)a.q1, (int8_t*)a.q2, K,
                                 (float*)a.alpha, a.a_step, 64, a.rg, s);
  if (rc) return rc;
  return launch_gemm_w8_mfma_probe(a, s);
}

int msd_probe_mfma_w4a16(const void* x_bf16, int64_t M, int64_t K, int64_t ldx, const uint8_t* W_fp4,
                         const uint8_t* W_e8m0, int64_t N, void* y, int out_dtype, int64_t ldy, void* workspace,
                         size_t workspace_bytes, const msd_debug_taps* /*taps*/, void* stream) {
  if (out_dtype != MSD_F32) return MSD_ERR_INVALID_ARG;
  if (M <= 0 || N <= 0 || K <= 0 || ldx < K || ldy < N || !gemm_w4_prefill_applies(M, K, N)) return MSD_ERR_SHAPE;
  if (!y || !x_bf16 || !W_fp4 || !W_e8m0) return MSD_ERR_INVALID_ARG;
  if (!aligned_to(W_fp4, 16) || !aligned_to(x_bf16, 2) || !aligned_to(y, 4)) return MSD_ERR_INVALID_ARG;
  const W4PrefillLayout l = w4_prefill_layout(M, K, N);
  if (l.total >= ((size_t)1 << 31)) return MSD_ERR_UNSUPPORTED;
  if (!workspace || !aligned_to(workspace, 256) || workspace_bytes < l.total) return MSD_ERR_WORKSPACE;
  return launch_gemm_w4_prefill((const uint16_t*)x_bf16, ldx, W_fp4, W_e8m0, y, 0, ldy, M, K, N, (uint8_t*)workspace,
                                MxVariant{}, (hipStream_t)stream, true);
}

size_t msd_dequant_gemm_workspace_bytes(int64_t M, int64_t K, int64_t N) {
  if (M <= 0 || K <= 0 || N <= 0) return 256;
  return dequant_workspace_bytes(M, K, N) + 256;
}

int msd_stream_read(const void* src, int64_t rows, int64_t row_bytes, void* stream) {
  if (rows < 0 || row_bytes < 0) return MSD_ERR_SHAPE;
  if (rows == 0) return MSD_OK;
  if (row_bytes == 0 || row_bytes % 256 != 0) return MSD_ERR_SHAPE;
  if (!src || !aligned_to(src, 16)) return MSD_ERR_INVALID_ARG;
  return launch_stream_read(src, rows, row_bytes, (hipStream_t)stream);
}

int msd_probe_mfma_rate(int fmt, const void* operands, int iters, void* stream) {
  if (fmt != MSD_INT8 && fmt != MSD_MXFP4) return MSD_ERR_INVALID_ARG;
  if (iters < 0 || iters > (1 << 22)) return MSD_ERR_SHAPE;
  if (!operands || !aligned_to(operands, 16)) return MSD_ERR_INVALID_ARG;
  return launch_mfma_rate(fmt == MSD_MXFP4, operands, iters, (hipStream_t)stream);
}

int msd_probe_lds_fill_rate(const void* src, int64_t src_bytes, int64_t hot_bytes, int hot_parts, int rounds,
                            void* stream) {
  if (src_bytes < 0 || hot_bytes < 0 || src_bytes % 1024 != 0 || hot_bytes % 1024 != 0) return MSD_ERR_SHAPE;
  if (hot_bytes < 1024 || src_bytes < hot_bytes + 1024 || src_bytes >= ((int64_t)1 << 46)) return MSD_ERR_SHAPE;
  if (hot_parts < 0 || hot_parts > 4 || rounds < 0 || rounds > (1 << 20)) return MSD_ERR_SHAPE;
  if (!src || !aligned_to(src, 16)) return MSD_ERR_INVALID_ARG;
  return launch_lds_fill_rate(src, src_bytes, hot_bytes, hot_parts, rounds, (hipStream_t)stream);
}

int msd_stream_read_linear(const void* src, int64_t bytes, void* stream) {
  if (bytes < 0 || bytes % 16 != 0 || bytes >= ((int64_t)1 << 46)) return MSD_ERR_SHAPE;
  if (bytes == 0) return MSD_OK;
  if (!src || !aligned_to(src, 16)) return MSD_ERR_INVALID_ARG;
  return launch_stream_read_linear(src, bytes, (hipStream_t)stream);
}

}  // extern "C"
