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
//   decode : 2M <= 64.  Up to four 16-row A fragments carry [x1; x2].  W goes HBM -> registers
//            in MFMA layout directly (each lane reads 16 contiguous bytes of one W row), the K
//            range is split over the waves of a workgroup and reduced through LDS.  For M <= 8
//            the kernel also decomposes the activations itself, under its own weight loads:
//            one launch per call and no code buffer in HBM.
//   tiled  : any M.  LDS-staged tiles, 4 waves, register-local merge of the two components.
#include <cstdlib>

#include "decompose_int8_dev.hpp"
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

// ------------------------------------------------------------------ decode (2M <= 16*RT)
// Every workgroup owns 16*NT output channels: each of its waves takes a contiguous K range,
// issues the loads of its W slice (HBM -> registers in MFMA B layout) FIRST, then obtains the
// matching A fragments and runs the MFMAs.  The wave partials are summed with LDS integer
// atomics (exact, order-independent).
//
// Where the A fragments come from:
//   SELF (M <= 8, one launch per call): the workgroup decomposes the activation rows itself
//       (Alg. 1 steps 1-5) while its weight loads are in flight -- the "online activation
//       decomposition" of Sec. 3.9; nothing is materialised in HBM.  Each wave reads the x
//       slice of its own K range (all rows), the row maxima are combined through LDS, then
//       the wave quantises its slice into wave-private LDS in A-fragment order.
//   otherwise: the codes were written to the workspace by the decomposition kernel.
//
// Bit-exact quantisation without a division per element.  q = rne(x/alpha) is computed as
// rne(x * (1/alpha)); the product differs from the correctly rounded quotient by at most
// 127*2^-22 < 3.1e-5 in absolute terms, so the two can round differently only if the product is
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

__device__ __forceinline__ void chunk_codes_fast(const Chunk16& c, float alpha, float ra, float beta,
                                                 float rb, uint4& o1, uint4& o2) {
  uint32_t a[4], b[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    uint32_t pa = 0, pb = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t w = c.w[j * 2 + (e >> 1)];
      const float x = (e & 1) ? __uint_as_float(w & 0xFFFF0000u) : __uint_as_float(w << 16);
      int c1, c2;
      int8_codes_fast(x, alpha, ra, beta, rb, c1, c2);
      pa |= ((uint32_t)c1 & 0xFFu) << (8 * e);
      pb |= ((uint32_t)c2 & 0xFFu) << (8 * e);
    }
    a[j] = pa;
    b[j] = pb;
  }
  o1 = make_uint4(a[0], a[1], a[2], a[3]);
  o2 = make_uint4(b[0], b[1], b[2], b[3]);
}

constexpr int kSelfMaxRows = 8;

template <int WAVES, int UNROLL, int RT, int NT, bool SELF>
__global__ __launch_bounds__(WAVES * 64) void gemm_w8_decode_kernel(GemmW8Args a) {
  constexpr int THREADS = WAVES * 64;
  __shared__ int s_acc[RT][NT][4][64];
  __shared__ float s_red[SELF ? kSelfMaxRows * WAVES : 1];
  __shared__ float s_alpha[kSelfMaxRows];
  extern __shared__ __attribute__((aligned(16))) int8_t s_codes[];  // SELF: per wave [2][M][kw]
  const int M = (int)a.M;
  const int64_t K = a.K, N = a.N;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int row = lane & 15, g = lane >> 4;
  for (int i = threadIdx.x; i < RT * NT * 256; i += THREADS) (&s_acc[0][0][0][0])[i] = 0;
  const int64_t n0 = (int64_t)blockIdx.x * (16 * NT);
  const int ksteps = (int)((K + 63) / 64);
  const int per = (ksteps + WAVES - 1) / WAVES;
  const int ks0 = min(wave * per, ksteps);
  const int ks1 = min(ksteps, ks0 + per);
  const int kw = per * 64;  // K range a wave can own (its LDS stride)
  const int8_t* wp[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) wp[t] = a.W + min(n0 + 16 * t + row, N - 1) * K + 16 * g;
  // A-fragment source of this lane: stacked row i = f*16 + row; [0,M) -> x1, [M,2M) -> x2
  int8_t* my_codes = s_codes + (int64_t)wave * 2 * M * kw;
  const int8_t* ap[RT];
#pragma unroll
  for (int f = 0; f < RT; ++f) {
    const int i = f * 16 + row;
    ap[f] = nullptr;
    if (SELF) {
      if (i < 2 * M) ap[f] = my_codes + (int64_t)i * kw + 16 * g - (int64_t)ks0 * 64;
    } else if (i < M) {
      ap[f] = a.q1 + (int64_t)i * a.ldq + 16 * g;
    } else if (i < 2 * M) {
      ap[f] = a.q2 + (int64_t)(i - M) * a.ldq + 16 * g;
    }
  }
  const v4i zero = {0, 0, 0, 0};
  v4i acc[RT][NT];
#pragma unroll
  for (int f = 0; f < RT; ++f)
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[f][t] = zero;
  bool ready = !SELF;
  float my_alpha = 0.f;  // SELF: alpha of row (threadIdx.x % kSelfMaxRows), kept for the epilogue
  for (int ks = ks0; ks < max(ks1, ks0 + 1); ks += UNROLL) {  // at least one pass: every wave joins the barriers
    v4i wv[NT][UNROLL], av[RT][UNROLL];
    bool ok[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int64_t k = (int64_t)(ks + u) * 64;
      ok[u] = (ks + u < ks1) && (k + 16 * g < K);
#pragma unroll
      for (int t = 0; t < NT; ++t) wv[t][u] = ok[u] ? ldg16_stream(wp[t] + k) : zero;
    }
    if (SELF && !ready) {
      // this wave's slice of x: rows [0,M) x columns [k_lo, k_hi), in chunks of 16 elements
      const int k_lo = ks0 * 64, k_hi = (int)min((int64_t)ks1 * 64, K);
      const int cpr = max(0, (k_hi - k_lo) / 16);  // chunks per row
      const int nch = M * cpr;
      const bool al16 = a.x_aligned != 0;
      // per-row maximum over the wave's slice (lane-private partials per row), then over the waves
      float mx[kSelfMaxRows];
#pragma unroll
      for (int m = 0; m < kSelfMaxRows; ++m) mx[m] = 0.f;
#pragma unroll 1
      for (int c = lane; c < nch; c += 64) {
        const int m = c / cpr;
        const float v = chunk_absmax(load_chunk16(a.x + (int64_t)m * a.ldx + k_lo + (c - m * cpr) * 16, al16));
#pragma unroll
        for (int mm = 0; mm < kSelfMaxRows; ++mm) mx[mm] = (m == mm) ? fmaxf(mx[mm], v) : mx[mm];
      }
#pragma unroll
      for (int m = 0; m < kSelfMaxRows; ++m) {
        const float v = m < M ? wave_max(mx[m]) : 0.f;
        if (lane == 0) s_red[m * WAVES + wave] = v;
      }
      __syncthreads();
      if (threadIdx.x < kSelfMaxRows) {
        float v = s_red[threadIdx.x * WAVES];
#pragma unroll
        for (int w = 1; w < WAVES; ++w) v = fmaxf(v, s_red[threadIdx.x * WAVES + w]);
        s_alpha[threadIdx.x] = __fdiv_rn(v, 127.0f);
      }
      __syncthreads();
      my_alpha = s_alpha[threadIdx.x % kSelfMaxRows];
      const bool exporter = blockIdx.x == 0 && a.export_codes;
#pragma unroll 1
      for (int c = lane; c < nch; c += 64) {
        const int m = c / cpr, cc = c - m * cpr;
        const float al = s_alpha[m];
        uint4 o1 = make_uint4(0, 0, 0, 0), o2 = o1;
        if (al > 0.f) {
          const float be = __fdiv_rn(al, 254.0f);
          chunk_codes_fast(load_chunk16(a.x + (int64_t)m * a.ldx + k_lo + cc * 16, al16), al,
                           __fdiv_rn(1.0f, al), be, __fdiv_rn(1.0f, be), o1, o2);
        }
        *reinterpret_cast<uint4*>(my_codes + (int64_t)m * kw + cc * 16) = o1;
        *reinterpret_cast<uint4*>(my_codes + (int64_t)(M + m) * kw + cc * 16) = o2;
        if (exporter) {  // observation points only
          *reinterpret_cast<uint4*>(const_cast<int8_t*>(a.q1) + (int64_t)m * a.ldq + k_lo + cc * 16) = o1;
          *reinterpret_cast<uint4*>(const_cast<int8_t*>(a.q2) + (int64_t)m * a.ldq + k_lo + cc * 16) = o2;
        }
      }
      if (exporter && threadIdx.x < M) const_cast<float*>(a.alpha)[threadIdx.x] = s_alpha[threadIdx.x];
      __builtin_amdgcn_wave_barrier();  // the codes are wave-private: no workgroup barrier needed
      ready = true;
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int64_t k = (int64_t)(ks + u) * 64;
#pragma unroll
      for (int f = 0; f < RT; ++f) av[f][u] = (ok[u] && ap[f]) ? ldg16(ap[f] + k) : zero;
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
#pragma unroll
      for (int f = 0; f < RT; ++f)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[f][t] = mfma16(av[f][u], wv[t][u], acc[f][t]);
  }
  __syncthreads();  // s_acc zeroed
  if (ks0 < ks1) {
#pragma unroll
    for (int f = 0; f < RT; ++f)
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) atomicAdd(&s_acc[f][t][r][lane], acc[f][t][r]);
  }
  __syncthreads();
  // thread e -> (tile t, column j, row m) with m fastest; stacked row i sits in fragment i/16,
  // register (i%16)%4 of lane ((i%16)/4)*16 + j
  const int mrows = SELF ? kSelfMaxRows : M;  // SELF: m = e % 8 = threadIdx.x % 8, matching my_alpha
  for (int e = threadIdx.x; e < mrows * 16 * NT; e += THREADS) {
    const int m = e % mrows, c = e / mrows;
    if (m >= M) continue;
    const int t = c >> 4, j = c & 15;
    const int i1 = m, i2 = M + m;
    const int a1 = s_acc[i1 >> 4][t][i1 & 3][((i1 & 15) >> 2) * 16 + j];
    const int a2 = s_acc[i2 >> 4][t][i2 & 3][((i2 & 15) >> 2) * 16 + j];
    const int64_t n = n0 + c;
    if (n < N) {
      const float alpha = SELF ? my_alpha : a.alpha[m];
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
constexpr int64_t kSelfMaxCodeBytes = 128 * 1024;  // LDS budget for the self-decomposed codes

// Single launch (the GEMM kernel decomposes the activations itself)?
bool gemm_w8_is_fused(int64_t M, int64_t K, int64_t) {
  // measured: beyond two rows the redundant per-workgroup decomposition costs more than a launch
  return M <= 2 && K > 0 && 2 * M * (K + 1024) <= kSelfMaxCodeBytes;
}

template <int WAVES, int UNROLL, int RT, int NT, bool SELF>
static int launch_decode(const GemmW8Args& a, hipStream_t stream) {
  const dim3 grid((unsigned)cdiv(a.N, 16 * NT));
  size_t dyn = 0;
  if (SELF) {
    const int64_t ksteps = (a.K + 63) / 64;
    const int64_t kw = cdiv(ksteps, WAVES) * 64;
    dyn = (size_t)(WAVES * 2 * a.M * kw);
    static size_t allowed = 0;  // per instantiation
    if (dyn > allowed) {
      MSD_HIP_CHECK(hipFuncSetAttribute(
          reinterpret_cast<const void*>(&gemm_w8_decode_kernel<WAVES, UNROLL, RT, NT, SELF>),
          hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSelfMaxCodeBytes));
      allowed = kSelfMaxCodeBytes;
    }
  }
  hipLaunchKernelGGL((gemm_w8_decode_kernel<WAVES, UNROLL, RT, NT, SELF>), grid, dim3(WAVES * 64), dyn, stream, a);
  return MSD_OK;
}

int launch_gemm_w8(const GemmW8Args& a, hipStream_t stream) {
  if (a.M == 0 || a.N == 0) return MSD_OK;
  const int64_t M = a.M, N = a.N;
  static const int tune = getenv("MSD_TUNE_W8") ? atoi(getenv("MSD_TUNE_W8")) : 0;
  int rc = MSD_OK;
  const bool wide = cdiv(N, 16) > 512;  // many column tiles: widen the workgroup tile (measured)
  (void)tune;
  if (a.x != nullptr) {  // the caller asked for the single-launch path (gemm_w8_is_fused)
    rc = launch_decode<4, 8, 1, 1, true>(a, stream);
  } else if (2 * M <= 16) {
    rc = wide ? launch_decode<4, 8, 1, 2, false>(a, stream) : launch_decode<4, 8, 1, 1, false>(a, stream);
  } else if (2 * M <= 32) {
    rc = launch_decode<8, 4, 2, 2, false>(a, stream);
  } else if (2 * M <= 64) {
    rc = wide ? launch_decode<8, 2, 4, 4, false>(a, stream) : launch_decode<8, 4, 4, 1, false>(a, stream);
  } else if (cdiv(M, 64) * cdiv(N, 128) < 256) {
    // few, tall tiles: narrow the N tile so that a decode-sized problem still covers the chip
    const dim3 grid((unsigned)cdiv(N, 32), (unsigned)cdiv(M, 64));
    hipLaunchKernelGGL((gemm_w8_tiled_kernel<64, 32, 4, 1>), grid, dim3(256), 0, stream, a);
  } else {
    const dim3 grid((unsigned)cdiv(N, 128), (unsigned)cdiv(M, 64));
    hipLaunchKernelGGL((gemm_w8_tiled_kernel<64, 128, 2, 2>), grid, dim3(256), 0, stream, a);
  }
  if (rc) return rc;
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

}  // namespace msd
