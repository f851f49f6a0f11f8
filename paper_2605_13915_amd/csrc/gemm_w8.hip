// W8A16 MSD GEMM for gfx950: dual INT8 MFMA products against the still-quantised weights
// and a dual-scale fp32 epilogue (paper Alg. 1 steps 6-8; fused tiled realisation, Sec. 3.9).
//
// Both activation components ride one pass over W: the rows of x1 and x2 are stacked into
// one left operand (the row-concatenation of Sec. 3.9), every weight fragment that reaches
// a register is multiplied by both, and y = s_W*(alpha*acc1 + beta*acc2) is formed in
// registers, so the int32 partial products never reach HBM.
//
// MFMA used: v_mfma_i32_16x16x64_i8.  Operand layout (lane l of 64): A holds row l%16,
// 16 consecutive k bytes of group l/16; B holds column l%16, same k bytes; D holds column
// l%16, rows 4*(l/16)+r in register r.  A = stacked activation codes, B = W rows.
//
// Two kernels:
//   skinny : 2M <= 64.  Up to four 16-row A fragments carry [x1; x2].  W goes HBM -> registers in
//            MFMA layout directly (each lane reads 16 contiguous bytes of one W row), the
//            K range is split over the waves of a workgroup and reduced through LDS.
//   tiled  : any M.  LDS-staged tiles, 4 waves, register-local merge of the two components.
#include "kernels.hpp"

namespace msd {

__device__ __forceinline__ v4i mfma16(v4i a, v4i b, v4i c) {
  return __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ v4i ldg16(const int8_t* p) {
  return *reinterpret_cast<const v4i*>(p);
}
// streaming load for weights that are read exactly once
__device__ __forceinline__ v4i ldg16_stream(const int8_t* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const v4i*>(p));
}

__device__ __forceinline__ void store_out(void* y, int out_bf16, int64_t idx, float v) {
  if (out_bf16)
    reinterpret_cast<uint16_t*>(y)[idx] = f32_to_bf16_bits(v);
  else
    reinterpret_cast<float*>(y)[idx] = v;
}

__device__ __forceinline__ float merge_scales(float sw, float alpha, float beta, int a1, int a2) {
  // y = s_W * (alpha*acc1 + beta*acc2)   (Alg. 1 step 8)
  return sw * (alpha * (float)a1 + beta * (float)a2);
}

// ------------------------------------------------------------------ skinny (2M <= 16*RT)
// One workgroup per 16 output channels.  The stacked rows [x1; x2] fill RT A fragments; each
// wave owns a contiguous K range, streams its 16 x (K/WAVES) slice of W from HBM straight into
// MFMA B fragments and reads the matching A fragments from the (cache-resident) code buffers.
template <int WAVES, int UNROLL, int RT>
__global__ __launch_bounds__(WAVES * 64) void gemm_w8_skinny_kernel(GemmW8Args a) {
  __shared__ int s_part[WAVES][RT][4][64];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int row = lane & 15, g = lane >> 4;
  const int M = (int)a.M;
  const int64_t K = a.K, N = a.N;
  const int64_t n0 = (int64_t)blockIdx.x * 16;
  const int ksteps = (int)((K + 63) / 64);
  const int per = (ksteps + WAVES - 1) / WAVES;
  const int ks0 = wave * per;
  const int ks1 = min(ksteps, ks0 + per);
  const int64_t wrow = min(n0 + row, N - 1);
  const int8_t* wp = a.W + wrow * K + 16 * g;
  const int8_t* ap[RT];
#pragma unroll
  for (int f = 0; f < RT; ++f) {
    const int i = f * 16 + row;  // stacked row: [0,M) -> x1, [M,2M) -> x2
    ap[f] = nullptr;
    if (i < M)
      ap[f] = a.q1 + (int64_t)i * a.ldq + 16 * g;
    else if (i < 2 * M)
      ap[f] = a.q2 + (int64_t)(i - M) * a.ldq + 16 * g;
  }
  const v4i zero = {0, 0, 0, 0};
  v4i acc[RT];
#pragma unroll
  for (int f = 0; f < RT; ++f) acc[f] = zero;
  for (int ks = ks0; ks < ks1; ks += UNROLL) {
    v4i wv[UNROLL], av[RT][UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int64_t k = (int64_t)(ks + u) * 64;
      const bool ok = (ks + u < ks1) && (k + 16 * g < K);
      wv[u] = ok ? ldg16_stream(wp + k) : zero;
#pragma unroll
      for (int f = 0; f < RT; ++f) av[f][u] = (ok && ap[f]) ? ldg16(ap[f] + k) : zero;
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
#pragma unroll
      for (int f = 0; f < RT; ++f) acc[f] = mfma16(av[f][u], wv[u], acc[f]);
  }
#pragma unroll
  for (int f = 0; f < RT; ++f)
#pragma unroll
    for (int r = 0; r < 4; ++r) s_part[wave][f][r][lane] = acc[f][r];
  __syncthreads();
  // thread t -> (m = t/16, j = t%16); stacked row i sits in fragment i/16, register (i%16)%4 of
  // lane ((i%16)/4)*16 + j
  for (int t = threadIdx.x; t < M * 16; t += WAVES * 64) {
    const int m = t >> 4, j = t & 15;
    const int i1 = m, i2 = M + m;
    int a1 = 0, a2 = 0;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
      a1 += s_part[w][i1 >> 4][i1 & 3][((i1 & 15) >> 2) * 16 + j];
      a2 += s_part[w][i2 >> 4][i2 & 3][((i2 & 15) >> 2) * 16 + j];
    }
    const int64_t n = n0 + j;
    if (n < N) {
      const float alpha = a.alpha[m];
      const float beta = __fdiv_rn(alpha, 254.0f);
      store_out(a.y, a.out_bf16, (int64_t)m * a.ldy + n, merge_scales(a.w_scale[n], alpha, beta, a1, a2));
      if (a.acc1) a.acc1[(int64_t)m * N + n] = a1;
      if (a.acc2) a.acc2[(int64_t)m * N + n] = a2;
    }
  }
}

// ------------------------------------------------------------------ tiled (any M)
// Workgroup tile: BMH activation rows (both components -> 2*BMH stacked rows) x BN weight
// rows, K step 64.  Waves are laid out WM x WN; each wave owns TMH = BMH/WM activation rows
// (both components, so the merge is register-local) and TN = BN/WN output channels.
constexpr int kBK = 64;
constexpr int kLdsStride = kBK + 16;  // +16 B: consecutive rows land in distinct 16 B bank groups

template <int BMH, int BN, int WM, int WN>
struct TiledCfg {
  static constexpr int kThreads = WM * WN * 64;
  static constexpr int kRowsA = 2 * BMH;
  static constexpr int kTMH = BMH / WM;
  static constexpr int kTN = BN / WN;
  static constexpr int kFragM = kTMH / 16;  // per component
  static constexpr int kFragN = kTN / 16;
  static constexpr int kChunksA = kRowsA * (kBK / 16);
  static constexpr int kChunksB = BN * (kBK / 16);
  static constexpr int kLdA = (kChunksA + kThreads - 1) / kThreads;
  static constexpr int kLdB = (kChunksB + kThreads - 1) / kThreads;
};

template <int BMH, int BN, int WM, int WN>
__global__ __launch_bounds__(WM * WN * 64) void gemm_w8_tiled_kernel(GemmW8Args a) {
  using C = TiledCfg<BMH, BN, WM, WN>;
  __shared__ __attribute__((aligned(16))) int8_t sA[C::kRowsA * kLdsStride];
  __shared__ __attribute__((aligned(16))) int8_t sB[BN * kLdsStride];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int row16 = lane & 15, g = lane >> 4;
  const int64_t M = a.M, K = a.K, N = a.N;
  const int64_t m0 = (int64_t)blockIdx.y * BMH;
  const int64_t n0 = (int64_t)blockIdx.x * BN;
  const int ks0 = 0;
  const int ks1 = (int)((K + kBK - 1) / kBK);
  const v4i zero = {0, 0, 0, 0};

  // global -> register staging of one K step
  v4i ra[C::kLdA], rb[C::kLdB];
  auto load_tiles = [&](int ks) {
    const int64_t k0 = (int64_t)ks * kBK;
#pragma unroll
    for (int i = 0; i < C::kLdA; ++i) {
      const int c = tid + i * C::kThreads;
      const int r = c >> 2, kc = (c & 3) * 16;
      v4i v = zero;
      if (c < C::kChunksA) {
        const int comp = r / BMH;
        const int64_t m = m0 + (r - comp * BMH);
        if (m < M && k0 + kc < K) v = ldg16((comp ? a.q2 : a.q1) + m * a.ldq + k0 + kc);
      }
      ra[i] = v;
    }
#pragma unroll
    for (int i = 0; i < C::kLdB; ++i) {
      const int c = tid + i * C::kThreads;
      const int r = c >> 2, kc = (c & 3) * 16;
      v4i v = zero;
      if (c < C::kChunksB) {
        const int64_t n = n0 + r;
        if (n < N && k0 + kc < K) v = ldg16_stream(a.W + n * K + k0 + kc);
      }
      rb[i] = v;
    }
  };
  auto store_tiles = [&]() {
#pragma unroll
    for (int i = 0; i < C::kLdA; ++i) {
      const int c = tid + i * C::kThreads;
      if (c < C::kChunksA) *reinterpret_cast<v4i*>(&sA[(c >> 2) * kLdsStride + (c & 3) * 16]) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < C::kLdB; ++i) {
      const int c = tid + i * C::kThreads;
      if (c < C::kChunksB) *reinterpret_cast<v4i*>(&sB[(c >> 2) * kLdsStride + (c & 3) * 16]) = rb[i];
    }
  };

  v4i acc[2][C::kFragM][C::kFragN];
#pragma unroll
  for (int c = 0; c < 2; ++c)
#pragma unroll
    for (int i = 0; i < C::kFragM; ++i)
#pragma unroll
      for (int j = 0; j < C::kFragN; ++j) acc[c][i][j] = zero;

  if (ks0 < ks1) load_tiles(ks0);
  for (int ks = ks0; ks < ks1; ++ks) {
    __syncthreads();  // previous step's LDS reads are done
    store_tiles();
    __syncthreads();
    if (ks + 1 < ks1) load_tiles(ks + 1);
    v4i fb[C::kFragN];
#pragma unroll
    for (int j = 0; j < C::kFragN; ++j)
      fb[j] = *reinterpret_cast<const v4i*>(&sB[(wn * C::kTN + 16 * j + row16) * kLdsStride + 16 * g]);
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int i = 0; i < C::kFragM; ++i) {
        const v4i fa = *reinterpret_cast<const v4i*>(
            &sA[(c * BMH + wm * C::kTMH + 16 * i + row16) * kLdsStride + 16 * g]);
#pragma unroll
        for (int j = 0; j < C::kFragN; ++j) acc[c][i][j] = mfma16(fa, fb[j], acc[c][i][j]);
      }
  }

  // ---- dual-scale epilogue
#pragma unroll
  for (int i = 0; i < C::kFragM; ++i)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int64_t m = m0 + wm * C::kTMH + 16 * i + 4 * g + r;
      if (m >= M) continue;
      const float alpha = a.alpha[m];
      const float beta = __fdiv_rn(alpha, 254.0f);
#pragma unroll
      for (int j = 0; j < C::kFragN; ++j) {
        const int64_t n = n0 + wn * C::kTN + 16 * j + row16;
        if (n >= N) continue;
        const int a1 = acc[0][i][j][r], a2 = acc[1][i][j][r];
        store_out(a.y, a.out_bf16, m * a.ldy + n, merge_scales(a.w_scale[n], alpha, beta, a1, a2));
        if (a.acc1) a.acc1[m * N + n] = a1;
        if (a.acc2) a.acc2[m * N + n] = a2;
      }
    }
}

// ------------------------------------------------------------------ dispatch
void gemm_w8_scratch(int64_t, int64_t, int64_t, size_t* part_bytes, size_t* counter_bytes) {
  *part_bytes = 0;
  *counter_bytes = 0;
}

int launch_gemm_w8(const GemmW8Args& a, hipStream_t stream) {
  if (a.M == 0 || a.N == 0) return MSD_OK;
  const int64_t M = a.M, N = a.N;
  if (2 * M <= 64) {
    const dim3 grid((unsigned)cdiv(N, 16));
    if (2 * M <= 16)
      hipLaunchKernelGGL((gemm_w8_skinny_kernel<8, 8, 1>), grid, dim3(512), 0, stream, a);
    else if (2 * M <= 32)
      hipLaunchKernelGGL((gemm_w8_skinny_kernel<8, 4, 2>), grid, dim3(512), 0, stream, a);
    else
      hipLaunchKernelGGL((gemm_w8_skinny_kernel<8, 4, 4>), grid, dim3(512), 0, stream, a);
  } else if (cdiv(M, 64) * cdiv(N, 128) < 256) {
    // few, tall tiles: narrow the N tile so that a decode-sized problem still covers the chip
    const dim3 grid((unsigned)cdiv(N, 32), (unsigned)cdiv(M, 64));
    hipLaunchKernelGGL((gemm_w8_tiled_kernel<64, 32, 4, 1>), grid, dim3(256), 0, stream, a);
  } else {
    const dim3 grid((unsigned)cdiv(N, 128), (unsigned)cdiv(M, 64));
    hipLaunchKernelGGL((gemm_w8_tiled_kernel<64, 128, 2, 2>), grid, dim3(256), 0, stream, a);
  }
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

}  // namespace msd
