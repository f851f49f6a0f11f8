// Comparison kernels: the conventional dequantise-then-BF16-GEMM path the paper argues
// against (Sec. 3.1 first equation; the "Dequant" rows of Sec. 6), written as the fused GPU
// form: the weight tile is read once from HBM, lifted to BF16 in registers
// (bf16(s_W * w) for INT8; the exact BF16 value 2^e * w for MXFP4) and multiplied with the
// BF16 activations on v_mfma_f32_16x16x32_bf16 with fp32 accumulation.  Same work split as
// the MSD skinny kernels (16 output channels per workgroup, K split over the waves), so the
// two paths differ only in what the paper changes: per-element weight conversion on the
// vector ALU and a BF16 instead of an INT8 / FP4 matrix instruction.  With 256 or more
// activation rows (and enough workspace) the two-step form at the end of this file runs instead.
#include "kernels.hpp"

namespace msd {

typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));

__device__ __forceinline__ v4f mfma_bf16(v8bf a, v8bf b, v4f c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {  // RNE, hardware convert
  const v2f f = {lo, hi};
  const v2bf b = __builtin_convertvector(f, v2bf);
  return *reinterpret_cast<const uint32_t*>(&b);
}

union Frag8 {
  uint32_t u[4];
  v8bf v;
};

// INT8: 16 weight bytes -> two fragments of 8 BF16 values bf16(scale * w)
__device__ __forceinline__ void dequant_i8x16(v4i w, float scale, Frag8 (&out)[2]) {
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const int x = w[d];
    const float f0 = scale * (float)(int)(int8_t)(x & 0xFF);
    const float f1 = scale * (float)(int)(int8_t)((x >> 8) & 0xFF);
    const float f2 = scale * (float)(int)(int8_t)((x >> 16) & 0xFF);
    const float f3 = scale * (float)(int)(int8_t)((x >> 24) & 0xFF);
    out[d >> 1].u[(d & 1) * 2 + 0] = pack_bf16(f0, f1);
    out[d >> 1].u[(d & 1) * 2 + 1] = pack_bf16(f2, f3);
  }
}

// MXFP4: one E2M1 nibble and the block exponent -> BF16 bits of 2^(e-127) * value (exact)
__device__ __forceinline__ uint32_t e2m1_to_bf16(uint32_t nib, int eadj) {
  // magnitudes 0, .5, 1, 1.5, 2, 3, 4, 6 as BF16: exponent field 126 + (m>>1) (m>=2), mantissa bit 6
  const uint32_t m = nib & 7u;
  if (m == 0) return 0;
  uint32_t bits;
  if (m == 1)
    bits = 0x3F00u;  // 0.5
  else
    bits = ((126u + (m >> 1)) << 7) | ((m & 1u) << 6);
  bits += (uint32_t)(eadj << 7);
  return bits | ((nib & 8u) << 12);
}

__device__ __forceinline__ void dequant_fp4x32(v4i w, int ebyte, Frag8 (&out)[4]) {
  const int eadj = ebyte - 127;
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const uint32_t x = (uint32_t)w[d];
#pragma unroll
    for (int pair = 0; pair < 4; ++pair) {
      const uint32_t lo = e2m1_to_bf16((x >> (8 * pair)) & 15u, eadj);
      const uint32_t hi = e2m1_to_bf16((x >> (8 * pair + 4)) & 15u, eadj);
      out[d].u[pair] = lo | (hi << 16);
    }
  }
}

struct DqArgs {
  const uint16_t* x;
  int64_t ldx;
  const uint8_t* W;   // int8 [N][K] or fp4 [N][K/2]
  const float* w_scale;  // INT8 only
  const uint8_t* We;     // MXFP4 only
  void* y;
  int out_bf16;
  int64_t ldy;
  int64_t M, K, N;
};

// FMT 8: INT8 weights, 64 k per wave step.  FMT 4: MXFP4 weights, 128 k per wave step.
template <int FMT, int WAVES, int RT>
__global__ __launch_bounds__(WAVES * 64) void dequant_gemm_kernel(DqArgs a) {
  constexpr int KSTEP = FMT == 8 ? 64 : 128;
  constexpr int KPL = KSTEP / 4;  // k values per lane per step
  constexpr int NF = KPL / 8;     // BF16 fragments per step
  __shared__ float s_part[WAVES][RT][4][64];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int row = lane & 15, g = lane >> 4;
  const int64_t M = a.M, K = a.K, N = a.N;
  const int64_t n0 = (int64_t)blockIdx.x * 16;
  const int64_t m0 = (int64_t)blockIdx.y * 16 * RT;
  const int64_t steps = (K + KSTEP - 1) / KSTEP;
  const int64_t per = (steps + WAVES - 1) / WAVES;
  const int64_t s0 = wave * per, s1 = min(steps, s0 + per);
  const int64_t wrow = min(n0 + row, N - 1);
  const float scale = FMT == 8 ? a.w_scale[wrow] : 0.f;
  v4f acc[RT];
#pragma unroll
  for (int f = 0; f < RT; ++f) acc[f] = v4f{0.f, 0.f, 0.f, 0.f};
  const v4i zero4 = {0, 0, 0, 0};
  for (int64_t s = s0; s < s1; ++s) {
    const int64_t k = s * KSTEP + KPL * g;  // first k of this lane
    const bool ok = k < K;                  // K % 16 (INT8) / K % 32 (MXFP4) == 0: all or nothing
    Frag8 wf[NF];
    if constexpr (FMT == 8) {
      const v4i w = ok ? __builtin_nontemporal_load(reinterpret_cast<const v4i*>(a.W + wrow * K + k)) : zero4;
      dequant_i8x16(w, scale, reinterpret_cast<Frag8(&)[2]>(wf));
    } else {
      const v4i w = ok ? __builtin_nontemporal_load(reinterpret_cast<const v4i*>(a.W + wrow * (K / 2) + k / 2)) : zero4;
      const int eb = ok ? (int)a.We[wrow * (K / 32) + k / 32] : 127;
      dequant_fp4x32(w, eb, reinterpret_cast<Frag8(&)[4]>(wf));
    }
#pragma unroll
    for (int f = 0; f < RT; ++f) {
      const int64_t m = m0 + 16 * f + row;
#pragma unroll
      for (int u = 0; u < NF; ++u) {
        Frag8 xf;
        const uint4 v = (ok && m < M) ? *reinterpret_cast<const uint4*>(a.x + m * a.ldx + k + 8 * u)
                                      : make_uint4(0, 0, 0, 0);
        xf.u[0] = v.x; xf.u[1] = v.y; xf.u[2] = v.z; xf.u[3] = v.w;
        acc[f] = mfma_bf16(xf.v, wf[u].v, acc[f]);
      }
    }
  }
#pragma unroll
  for (int f = 0; f < RT; ++f)
#pragma unroll
    for (int r = 0; r < 4; ++r) s_part[wave][f][r][lane] = acc[f][r];
  __syncthreads();
  for (int t = threadIdx.x; t < RT * 256; t += WAVES * 64) {
    const int i = t >> 4, j = t & 15;
    const int64_t m = m0 + i, n = n0 + j;
    if (m >= M || n >= N) continue;
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) v += s_part[w][i >> 4][i & 3][((i & 15) >> 2) * 16 + j];
    if (a.out_bf16)
      reinterpret_cast<uint16_t*>(a.y)[m * a.ldy + n] = f32_to_bf16_bits(v);
    else
      reinterpret_cast<float*>(a.y)[m * a.ldy + n] = v;
  }
}

template <int FMT>
static int launch_dq(const DqArgs& a, hipStream_t stream) {
  if (a.M <= 16)
    hipLaunchKernelGGL((dequant_gemm_kernel<FMT, 8, 1>), dim3((unsigned)cdiv(a.N, 16), 1), dim3(512), 0, stream, a);
  else if (a.M <= 32)
    hipLaunchKernelGGL((dequant_gemm_kernel<FMT, 8, 2>), dim3((unsigned)cdiv(a.N, 16), 1), dim3(512), 0, stream, a);
  else
    hipLaunchKernelGGL((dequant_gemm_kernel<FMT, 8, 4>), dim3((unsigned)cdiv(a.N, 16), (unsigned)cdiv(a.M, 64)),
                       dim3(512), 0, stream, a);
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

// ------------------------------------------------------------------ prefill: dequantise, then GEMM
// For many activation rows the comparison path is the literal two-step form: one pass lifts the
// whole weight matrix to BF16 in HBM (bf16(s_W * w), or the exact MXFP4 value), then a BF16 GEMM
// runs on the same asynchronous-fill pipeline as the MSD prefill kernel (launch_bf16_gemm_tiled),
// so that both paths get the same engineering.  Needs 2*N*K bytes of workspace.
constexpr int64_t kTiledMinRows = 256;

__global__ __launch_bounds__(256) void dequant_w8_to_bf16_kernel(const int8_t* __restrict__ W,
                                                                 const float* __restrict__ w_scale, int64_t N,
                                                                 int64_t K, uint16_t* __restrict__ out) {
  const int64_t chunks = K / 16;  // 16 weights per thread
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= N * chunks) return;
  const int64_t n = gid / chunks;
  const v4i w = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(W) + gid);
  Frag8 f[2];
  dequant_i8x16(w, w_scale[n], f);
  uint4* o = reinterpret_cast<uint4*>(out + gid * 16);
  o[0] = make_uint4(f[0].u[0], f[0].u[1], f[0].u[2], f[0].u[3]);
  o[1] = make_uint4(f[1].u[0], f[1].u[1], f[1].u[2], f[1].u[3]);
}

__global__ __launch_bounds__(256) void dequant_w4_to_bf16_kernel(const uint8_t* __restrict__ W,
                                                                 const uint8_t* __restrict__ We, int64_t blocks,
                                                                 uint16_t* __restrict__ out) {
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;  // one 32-element block per thread
  if (gid >= blocks) return;
  const v4i w = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(W) + gid);
  Frag8 f[4];
  dequant_fp4x32(w, (int)We[gid], f);
  uint4* o = reinterpret_cast<uint4*>(out + gid * 32);
#pragma unroll
  for (int i = 0; i < 4; ++i) o[i] = make_uint4(f[i].u[0], f[i].u[1], f[i].u[2], f[i].u[3]);
}

size_t dequant_workspace_bytes(int64_t M, int64_t K, int64_t N) {
  return M >= kTiledMinRows ? align_up((size_t)N * K * 2, 256) : 0;
}

static bool use_tiled(int64_t M, int64_t K, const uint16_t* x, int64_t ldx, void* ws, size_t ws_bytes, int64_t N) {
  return M >= kTiledMinRows && K % 32 == 0 && K > 0 && ws != nullptr && ws_bytes >= (size_t)N * K * 2 &&
         (reinterpret_cast<uintptr_t>(x) & 15) == 0 && ldx % 8 == 0 && (reinterpret_cast<uintptr_t>(ws) & 15) == 0;
}

int launch_dequant_gemm_w8(const uint16_t* x, int64_t M, int64_t K, int64_t ldx, const int8_t* W,
                           const float* w_scale, int64_t N, void* y, int out_bf16, int64_t ldy, void* ws,
                           size_t ws_bytes, hipStream_t stream) {
  if (use_tiled(M, K, x, ldx, ws, ws_bytes, N)) {
    uint16_t* Wb = reinterpret_cast<uint16_t*>(ws);
    const int64_t items = N * (K / 16);
    hipLaunchKernelGGL(dequant_w8_to_bf16_kernel, dim3((unsigned)cdiv(items, 256)), dim3(256), 0, stream, W,
                       w_scale, N, K, Wb);
    MSD_LAUNCH_CHECK();
    return launch_bf16_gemm_tiled(x, M, K, ldx, Wb, N, y, out_bf16, ldy, stream);
  }
  DqArgs a{x, ldx, (const uint8_t*)W, w_scale, nullptr, y, out_bf16, ldy, M, K, N};
  return launch_dq<8>(a, stream);
}

int launch_dequant_gemm_w4(const uint16_t* x, int64_t M, int64_t K, int64_t ldx, const uint8_t* W,
                           const uint8_t* We, int64_t N, void* y, int out_bf16, int64_t ldy, void* ws,
                           size_t ws_bytes, hipStream_t stream) {
  if (use_tiled(M, K, x, ldx, ws, ws_bytes, N)) {
    uint16_t* Wb = reinterpret_cast<uint16_t*>(ws);
    const int64_t blocks = N * (K / 32);
    hipLaunchKernelGGL(dequant_w4_to_bf16_kernel, dim3((unsigned)cdiv(blocks, 256)), dim3(256), 0, stream, W, We,
                       blocks, Wb);
    MSD_LAUNCH_CHECK();
    return launch_bf16_gemm_tiled(x, M, K, ldx, Wb, N, y, out_bf16, ldy, stream);
  }
  DqArgs a{x, ldx, W, nullptr, We, y, out_bf16, ldy, M, K, N};
  return launch_dq<4>(a, stream);
}

}  // namespace msd
