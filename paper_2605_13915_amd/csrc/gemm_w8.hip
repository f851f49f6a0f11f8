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
// Kernels:
//   decode : 2M <= 64.  Up to four 16-row A fragments carry [x1; x2].  W goes HBM -> registers
//            in MFMA layout directly (each lane reads 16 contiguous bytes of one W row), the K
//            range is split over the waves of a workgroup and reduced through LDS.  The codes come
//            from the decomposition launch in fragment-major order (one contiguous kilobyte per
//            operand load).
//   fused  : a handful of rows (M*K <= 16384).  The kernel also decomposes the activations itself,
//            under its own weight loads, all of which are in flight before any arithmetic starts:
//            one launch per call and no code buffer in HBM.
//   large  : any M.  32x32x32 MFMA, LDS-staged tiles (swizzled), 4 waves, register-local merge
//            of the two components; for prefill-sized problems a 256x256 tile filled by
//            asynchronous global->LDS loads four stages deep.
#include <type_traits>

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
// the same for the large-tile epilogues: the output is written once and not read again by the kernel
__device__ __forceinline__ void store_out_stream(void* y, int out_bf16, int64_t idx, float v) {
  if (out_bf16)
    __builtin_nontemporal_store(f32_to_bf16_bits(v), reinterpret_cast<uint16_t*>(y) + idx);
  else
    __builtin_nontemporal_store(v, reinterpret_cast<float*>(y) + idx);
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
//   SELF (one launch per call; the general single-launch form, chosen for M <= 2 when K has no instance of
//       the everything-in-flight kernel below): the workgroup decomposes the activation rows itself
//       (Alg. 1 steps 1-5) while its weight loads are in flight -- the "online activation
//       decomposition" of Sec. 3.9; nothing is materialised in HBM.  Each wave reads the x
//       slice of its own K range (all rows), the row maxima are combined through LDS, then
//       the wave quantises its slice into wave-private LDS in A-fragment order.
//   otherwise: the codes were written to the workspace by the decomposition kernel, fragment-major
//       (GemmW8Args::a_frag: one contiguous kilobyte per operand load) or, when observation points are
//       requested, row-major.
//
//   (the quantiser itself, bit-exact without a division per element, is in decompose_int8_dev.hpp)
constexpr int kSelfMaxRows = 8;
// rows the single-launch kernel accepts (measured: 16 x 1024 is slower than two launches, as 4 waves x 4 steps and
// as 16 waves x 1 step alike: the decomposition every workgroup repeats is bound by the CU's vector rate)
constexpr int kFusedMaxRows = 8;
constexpr int64_t kFusedMaxElems = 16384;  // ... and activation elements (M*K): beyond, a launch is cheaper
constexpr int64_t kSelfMaxCodeBytes = 136 * 1024;  // LDS budget for the self-decomposed codes

// FAST: K % 64 == 0, so no load of the main loop is predicated per lane (predicated loads do not
// batch); fragment rows past 2M then re-read row 0 -- their products are never looked at.
// SEG (canonical weights, FAST, every wave's K range a whole number of 256-byte segments): a B-operand load straight
// from [N][K] touches 16 weight rows with 64 bytes each; instead a wave fetches 256 contiguous bytes of a row per
// 16 lanes (four rows per instruction, four instructions per tile and four K steps) and turns them into operand
// order through 4 KB of LDS of its own per tile: chunk c of row r at chunk position c ^ r, so that the stores (eight
// consecutive lanes = half a row segment) and the operand reads (sixteen rows at one chunk) are conflict-free; no
// barrier, the LDS serves a wave in order.
template <int WAVES, int UNROLL, int RT, int NT, bool SELF, bool FAST, bool SEG = false>
__device__ __forceinline__ void gemm_w8_decode_body(const GemmW8Args& a, const int64_t n0) {
  constexpr int THREADS = WAVES * 64;
  static_assert(!SEG || (FAST && !SELF && UNROLL % 4 == 0), "row segments cover four K steps");
  __shared__ __attribute__((aligned(16))) int8_t s_seg[SEG ? WAVES * 4096 : 16];
  __shared__ int s_acc[RT][NT][4][64];
  __shared__ float s_red[SELF ? kSelfMaxRows * WAVES : 1];
  __shared__ float s_alpha[kSelfMaxRows];
  extern __shared__ __attribute__((aligned(16))) int8_t s_codes[];  // SELF: per wave [2][M][kw]
  const int M = (int)a.M;
  const int64_t K = a.K, N = a.N;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int row = lane & 15, g = lane >> 4;
  for (int i = threadIdx.x; i < RT * NT * 256; i += THREADS) (&s_acc[0][0][0][0])[i] = 0;
  const int ksteps = (int)((K + 63) / 64);
  const int per = (ksteps + WAVES - 1) / WAVES;
  const int ks0 = min(wave * per, ksteps);
  const int ks1 = min(ksteps, ks0 + per);
  const int kw = per * 64;  // K range a wave can own (its LDS stride)
  const int8_t* wp[NT];
  // packed weights: channel tile nb, K step ks at ((ks * tiles) + nb) kilobytes, the lane's 16 bytes at lane*16
  const int64_t wtiles = (N + 15) / 16;
  const int64_t wstep = a.w_packed ? wtiles * 1024 : 64;  // bytes between K steps of this lane's weight stream
#pragma unroll
  for (int t = 0; t < NT; ++t)
    wp[t] = a.w_packed ? a.W + min(n0 / 16 + t, wtiles - 1) * 1024 + lane * 16
                       : a.W + min(n0 + 16 * t + row, N - 1) * K + 16 * g;
  // SEG: instruction j of a group of four K steps covers rows 4 j .. 4 j + 3 of the tile, 16 lanes per row
  const int8_t* wseg[SEG ? NT : 1][4];
  int8_t* my_seg = s_seg + (SEG ? wave * 4096 : 0);
  if constexpr (SEG) {
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int j = 0; j < 4; ++j) wseg[t][j] = a.W + min(n0 + 16 * t + 4 * j + (lane >> 4), N - 1) * K + 16 * (lane & 15);
  }
  // A-fragment source of this lane: stacked row i = f*16 + row; [0,M) -> x1, [M,2M) -> x2
  int8_t* my_codes = s_codes + (int64_t)wave * 2 * M * kw;
  const int8_t* ap[RT];
#pragma unroll
  for (int f = 0; f < RT; ++f) {
    const int i = (FAST && f * 16 + row >= 2 * M) ? 0 : f * 16 + row;
    ap[f] = nullptr;
    if (SELF) {
      if (i < 2 * M) ap[f] = my_codes + (int64_t)i * kw + 16 * g - (int64_t)ks0 * 64;
    } else if (a.a_frag) {
      ap[f] = a.q1 + f * 1024 + lane * 16;  // rows past 2M hold whatever was there: their products are never read
    } else if (i < M) {
      ap[f] = a.q1 + (int64_t)i * a.ldq + 16 * g;
    } else if (i < 2 * M) {
      ap[f] = a.q2 + (int64_t)(i - M) * a.ldq + 16 * g;
    }
  }
  // bytes between the K steps of an A fragment (fragment-major codes: RT kilobyte blocks per step)
  const int64_t astep = (!SELF && a.a_frag) ? (int64_t)RT * 1024 : 64;
  const v4i zero = {0, 0, 0, 0};
  v4i acc[RT][NT];
#pragma unroll
  for (int f = 0; f < RT; ++f)
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[f][t] = zero;
  bool ready = !SELF;
  float my_alpha = 0.f;  // SELF: alpha of row (threadIdx.x % kSelfMaxRows), kept for the epilogue
  // scale factors of this thread's first output: requested now, needed after the last barrier
  const int rows_pre = SELF ? kSelfMaxRows : M;
  const int m_pre = (int)threadIdx.x % rows_pre;
  const int64_t n_pre = n0 + (int)threadIdx.x / rows_pre;
  const bool has_pre = (int)threadIdx.x < rows_pre * 16 * NT && m_pre < M && n_pre < N;
  const float ws_pre = has_pre ? a.w_scale[n_pre] : 0.f;
  const float alpha_pre = (!SELF && has_pre) ? a.alpha[m_pre] : 0.f;
  for (int ks = ks0; ks < max(ks1, ks0 + 1); ks += UNROLL) {  // at least one pass: every wave joins the barriers
    v4i wv[NT][UNROLL], av[RT][UNROLL];
    bool ok[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int64_t k = (int64_t)(ks + u) * 64;
      ok[u] = (ks + u < ks1) && (FAST || k + 16 * g < K);
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        wv[t][u] = zero;
        if constexpr (SEG) {  // register u of a group: rows 4 (u % 4) .., the 256 bytes of K steps ks + u - u % 4 ..
          if (ok[u]) wv[t][u] = ldg16_stream(wseg[t][u & 3] + (int64_t)(ks + (u & ~3)) * 64);
        } else {
          if (ok[u]) wv[t][u] = ldg16_stream(wp[t] + (ks + u) * wstep);
        }
      }
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
        s_alpha[threadIdx.x] = __fdiv_rn(v, a.rg.num1);
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
          const float be = __fdiv_rn(al, a.rg.num2);
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
#pragma unroll
      for (int f = 0; f < RT; ++f) {
        av[f][u] = zero;
        if (ok[u] && (FAST || ap[f])) av[f][u] = ldg16(ap[f] + (ks + u) * astep);
      }
    }
    if constexpr (SEG) {
#pragma unroll
      for (int q = 0; q < UNROLL / 4; ++q) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {  // one tile at a time through the wave's 4 KB
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int r = 4 * j + (lane >> 4), c = lane & 15;
            *reinterpret_cast<v4i*>(my_seg + r * 256 + ((c ^ r) & 15) * 16) = wv[t][4 * q + j];
          }
          __builtin_amdgcn_wave_barrier();
#pragma unroll
          for (int sub = 0; sub < 4; ++sub) {
            const v4i bf = *reinterpret_cast<const v4i*>(my_seg + row * 256 + (((4 * sub + g) ^ row) & 15) * 16);
#pragma unroll
            for (int f = 0; f < RT; ++f) acc[f][t] = mfma16(av[f][4 * q + sub], bf, acc[f][t]);
          }
          __builtin_amdgcn_wave_barrier();
        }
      }
    } else {
#pragma unroll
      for (int u = 0; u < UNROLL; ++u)
#pragma unroll
        for (int f = 0; f < RT; ++f)
#pragma unroll
          for (int t = 0; t < NT; ++t) acc[f][t] = mfma16(av[f][u], wv[t][u], acc[f][t]);
    }
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
      const bool first = e == (int)threadIdx.x;
      const float alpha = SELF ? my_alpha : first ? alpha_pre : a.alpha[m];
      const float beta = __fdiv_rn(alpha, a.rg.num2);
      const float ws = first ? ws_pre : a.w_scale[n];
      store_out(a.y, a.out_bf16, (int64_t)m * a.ldy + n, merge_scales(ws, alpha, beta, a1, a2));
      if (a.acc1) a.acc1[(int64_t)m * N + n] = a1;
      if (a.acc2) a.acc2[(int64_t)m * N + n] = a2;
    }
  }
}

template <int WAVES, int UNROLL, int RT, int NT, bool SELF, bool FAST, bool SEG = false>
__global__ __launch_bounds__(WAVES * 64) void gemm_w8_decode_kernel(GemmW8Args a) {
  gemm_w8_decode_body<WAVES, UNROLL, RT, NT, SELF, FAST, SEG>(a, (int64_t)blockIdx.x * (16 * NT));
}

// Grouped form for mixture-of-experts layers (paper Sec. 7.5: the decomposition is per activation
// row, so a grouped GEMM is the same computation per expert).  Rows are sorted by expert; expert
// e = blockIdx.y owns rows [offs[e], offs[e+1]) and its own weight matrix and scales.  The
// workgroup reads its expert's row range on the device (no host synchronisation), skips empty
// experts, and runs the decode body on chunks of 8*RT rows.
template <int WAVES, int UNROLL, int RT, int NT, bool FAST, bool SEG = false>
__global__ __launch_bounds__(WAVES * 64) void gemm_w8_grouped_kernel(GemmW8Args a, const int32_t* __restrict__ offs) {
  const int e = blockIdx.y;
  // a.M is the total number of rows: offsets outside [0, M] (a malformed routing table) are clamped, so
  // that no row index leaves the activation and output arrays
  const int64_t r1 = min((int64_t)offs[e + 1], a.M), r0 = max((int64_t)offs[e], (int64_t)0);
  const int64_t n0 = (int64_t)blockIdx.x * (16 * NT);
  for (int64_t c0 = r0; c0 < r1; c0 += 8 * RT) {
    GemmW8Args b = a;
    b.q1 = a.q1 + c0 * a.ldq;
    b.q2 = a.q2 + c0 * a.ldq;
    b.alpha = a.alpha + c0;
    b.W = a.W + (int64_t)e * a.N * a.K;
    b.w_scale = a.w_scale + (int64_t)e * a.N;
    b.y = a.out_bf16 ? (void*)(reinterpret_cast<uint16_t*>(a.y) + c0 * a.ldy)
                     : (void*)(reinterpret_cast<float*>(a.y) + c0 * a.ldy);
    b.M = min((int64_t)(8 * RT), r1 - c0);
    gemm_w8_decode_body<WAVES, UNROLL, RT, NT, false, FAST, SEG>(b, n0);
    __syncthreads();  // the accumulators in LDS are zeroed again by the next chunk
  }
}

// The decode body on chunks of 8*RT rows over blockIdx.y, all against the same weights: for 17..32 rows and
// few output channels a workgroup then pulls 16 rows of both components and 16*NT weight rows instead of all
// rows and 16 weight rows -- less L2 traffic per CU at the same number of workgroups.
template <int WAVES, int UNROLL, int RT, int NT, bool FAST>
__global__ __launch_bounds__(WAVES * 64) void gemm_w8_rowsplit_kernel(GemmW8Args a) {
  const int64_t c0 = (int64_t)blockIdx.y * (8 * RT);
  const int64_t n0 = (int64_t)blockIdx.x * (16 * NT);
  GemmW8Args b = a;
  b.q1 = a.q1 + c0 * a.ldq;
  b.q2 = a.q2 + c0 * a.ldq;
  b.alpha = a.alpha + c0;
  b.y = a.out_bf16 ? (void*)(reinterpret_cast<uint16_t*>(a.y) + c0 * a.ldy)
                   : (void*)(reinterpret_cast<float*>(a.y) + c0 * a.ldy);
  if (a.acc1) b.acc1 = a.acc1 + c0 * a.N;
  if (a.acc2) b.acc2 = a.acc2 + c0 * a.N;
  b.M = min((int64_t)(8 * RT), a.M - c0);
  gemm_w8_decode_body<WAVES, UNROLL, RT, NT, false, FAST>(b, n0);
}

// ------------------------------------------------------------------ single launch, everything in flight at once
// For a handful of rows (M <= MR, M*K <= kFusedMaxElems) and K = WAVES * STEPS * 64: a workgroup owns 16*NT
// output channels, wave w the K range [w, w+1) * STEPS * 64.  Each wave first requests its slice of x (all rows;
// it comes from L2), then its whole slice of W (STEPS * NT 16-byte loads per lane, HBM -> registers in MFMA B
// layout), so that every weight byte of the call is in flight before any arithmetic starts -- at these sizes the
// weight matrix is only a few times the bytes the memory system must have outstanding to run at its rate.
// Under those loads the workgroup decomposes the rows (Alg. 1 steps 1-5; the "online activation decomposition"
// of Sec. 3.9): row maxima over the waves through LDS, then each wave quantises its own slice into wave-private
// LDS (row pitch KW + 16 B: the 16 rows of an A fragment fall into 16 different 16-byte bank groups).  The
// MFMAs then take A from LDS and B from the registers the loads filled; wave partials meet in LDS integer
// atomics (exact).  Every workgroup repeats the decomposition, which is why the row count is bounded by work:
// at 16384 elements (about 18 vector instructions each) it costs about as much as the launch it saves.
// MR: compile-time bound on the rows (chunks of x held per lane: MR * STEPS / 16, at most 4).
// SEG: canonical weights fetched as 256-byte row segments and turned into operand order through 4 KB of LDS per
// wave, as in gemm_w8_decode_body.
template <int WAVES, int STEPS, int NT, int MR, bool SEG = false>
__global__ __launch_bounds__(WAVES * 64) void gemm_w8_fused_kernel(GemmW8Args a) {
  constexpr int THREADS = WAVES * 64, KW = STEPS * 64, CPR = KW / 16, PITCH = KW + 16;
  static_assert(!SEG || STEPS % 4 == 0, "row segments cover four K steps");
  __shared__ __attribute__((aligned(16))) int8_t s_seg[SEG ? WAVES * 4096 : 16];
  constexpr int XC = (MR * CPR + 63) / 64;
  constexpr int RT = (2 * MR + 15) / 16;
  static_assert(MR <= kFusedMaxRows && (CPR & (CPR - 1)) == 0 && XC <= 4, "rows / K range");
  __shared__ int s_acc[RT][NT][4][64];
  __shared__ float s_red[kFusedMaxRows][WAVES];
  __shared__ float s_par[kFusedMaxRows][4];  // alpha, 1/alpha, beta, 1/beta of each row
  extern __shared__ __attribute__((aligned(16))) int8_t s_codes[];  // per wave [2M][PITCH]
  const int M = (int)a.M;
  const int64_t K = a.K, N = a.N;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int row = lane & 15, g = lane >> 4;
  const int64_t n0 = (int64_t)blockIdx.x * (16 * NT);
  const int k_lo = wave * KW;
  // ---- x first (its loads are the oldest, so waiting for them does not wait for W)
  Chunk16 xc[XC];
  const bool al16 = a.x_aligned != 0;
  const int nch = M * CPR;
#pragma unroll
  for (int i = 0; i < XC; ++i) {
    const int c = lane + 64 * i;
    if (c < nch) {
      xc[i] = load_chunk16(a.x + (int64_t)(c / CPR) * a.ldx + k_lo + (c % CPR) * 16, al16);
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) xc[i].w[j] = 0;
    }
  }
  // ---- then the whole W slice of this wave
  v4i wv[NT][STEPS];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int64_t wtiles = (N + 15) / 16;
    const int8_t* wp = a.w_packed ? a.W + ((int64_t)wave * STEPS * wtiles + min(n0 / 16 + t, wtiles - 1)) * 1024 + lane * 16
                                  : a.W + min(n0 + 16 * t + row, N - 1) * K + k_lo + 16 * g;
    const int64_t wstep = a.w_packed ? wtiles * 1024 : 64;
    if constexpr (SEG) {  // register 4 q + j: rows 4 j .. 4 j + 3 of the tile, the 256 bytes of K steps 4 q .. 4 q + 3
#pragma unroll
      for (int s = 0; s < STEPS; ++s)
        wv[t][s] = ldg16_stream(a.W + min(n0 + 16 * t + 4 * (s & 3) + (lane >> 4), N - 1) * K + k_lo + (s >> 2) * 256 +
                                16 * (lane & 15));
    } else {
#pragma unroll
      for (int s = 0; s < STEPS; ++s) wv[t][s] = ldg16_stream(wp + s * wstep);
    }
  }
  // the weight scale of this thread's first output: requested now, needed after the last barrier
  const int64_t n_pre = n0 + (int)threadIdx.x / M;
  const float ws_pre = ((int)threadIdx.x < M * 16 * NT && n_pre < N) ? a.w_scale[n_pre] : 0.f;
  for (int i = threadIdx.x; i < RT * NT * 256; i += THREADS) (&s_acc[0][0][0][0])[i] = 0;
  // ---- row maxima: over the chunks of a lane, the lanes of a wave, the waves
  float cm[XC];
#pragma unroll
  for (int i = 0; i < XC; ++i) cm[i] = chunk_absmax(xc[i]);
#pragma unroll
  for (int m = 0; m < MR; ++m) {
    if (m < M) {
      float v = 0.f;
#pragma unroll
      for (int i = 0; i < XC; ++i) v = ((lane + 64 * i) / CPR == m) ? fmaxf(v, cm[i]) : v;
      v = wave_max(v);
      if (lane == 0) s_red[m][wave] = v;
    }
  }
  __syncthreads();
  if (threadIdx.x < M) {
    float v = s_red[threadIdx.x][0];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) v = fmaxf(v, s_red[threadIdx.x][w]);
    const float al = __fdiv_rn(v, a.rg.num1), be = __fdiv_rn(al, a.rg.num2);
    s_par[threadIdx.x][0] = al;
    s_par[threadIdx.x][1] = __fdiv_rn(1.0f, al);  // unused for an all-zero row
    s_par[threadIdx.x][2] = be;
    s_par[threadIdx.x][3] = __fdiv_rn(1.0f, be);
  }
  __syncthreads();
  // ---- quantise this wave's slice into its own LDS region
  int8_t* my_codes = s_codes + (int64_t)wave * 2 * M * PITCH;
  const bool exporter = blockIdx.x == 0 && a.export_codes;
#pragma unroll
  for (int i = 0; i < XC; ++i) {
    const int c = lane + 64 * i;
    if (c < nch) {
      const int m = c / CPR, cc = c % CPR;
      const float al = s_par[m][0];
      uint4 o1 = make_uint4(0, 0, 0, 0), o2 = o1;
      if (al > 0.f) chunk_codes_fast(xc[i], al, s_par[m][1], s_par[m][2], s_par[m][3], o1, o2);
      *reinterpret_cast<uint4*>(my_codes + m * PITCH + cc * 16) = o1;
      *reinterpret_cast<uint4*>(my_codes + (M + m) * PITCH + cc * 16) = o2;
      if (exporter) {  // observation points only
        *reinterpret_cast<uint4*>(const_cast<int8_t*>(a.q1) + (int64_t)m * a.ldq + k_lo + cc * 16) = o1;
        *reinterpret_cast<uint4*>(const_cast<int8_t*>(a.q2) + (int64_t)m * a.ldq + k_lo + cc * 16) = o2;
      }
    }
  }
  if (exporter && threadIdx.x < M) const_cast<float*>(a.alpha)[threadIdx.x] = s_par[threadIdx.x][0];
  __builtin_amdgcn_wave_barrier();  // the codes are wave-private: no workgroup barrier needed
  // ---- MFMAs: stacked row i of the A operand is x1 row i for i < M, x2 row i - M for i < 2M; rows past
  // that repeat row 0 (their products are never read)
  const v4i zero = {0, 0, 0, 0};
  v4i acc[RT][NT];
  const int8_t* afrag[RT];
#pragma unroll
  for (int f = 0; f < RT; ++f) {
    const int i = f * 16 + row;
    afrag[f] = my_codes + (i < 2 * M ? i : 0) * PITCH + 16 * g;
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[f][t] = zero;
  }
  if constexpr (SEG) {
    int8_t* my_seg = s_seg + wave * 4096;
#pragma unroll
    for (int q = 0; q < STEPS / 4; ++q)
#pragma unroll
      for (int t = 0; t < NT; ++t) {  // one tile at a time through the wave's 4 KB
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int r = 4 * j + (lane >> 4), c = lane & 15;
          *reinterpret_cast<v4i*>(my_seg + r * 256 + ((c ^ r) & 15) * 16) = wv[t][4 * q + j];
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int sub = 0; sub < 4; ++sub) {
          const v4i bf = *reinterpret_cast<const v4i*>(my_seg + row * 256 + (((4 * sub + g) ^ row) & 15) * 16);
#pragma unroll
          for (int f = 0; f < RT; ++f)
            acc[f][t] = mfma16(*reinterpret_cast<const v4i*>(afrag[f] + (4 * q + sub) * 64), bf, acc[f][t]);
        }
        __builtin_amdgcn_wave_barrier();
      }
  } else {
#pragma unroll
    for (int s = 0; s < STEPS; ++s) {
#pragma unroll
      for (int f = 0; f < RT; ++f) {
        const v4i av = *reinterpret_cast<const v4i*>(afrag[f] + s * 64);
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[f][t] = mfma16(av, wv[t][s], acc[f][t]);
      }
    }
  }
#pragma unroll
  for (int f = 0; f < RT; ++f)
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) atomicAdd(&s_acc[f][t][r][lane], acc[f][t][r]);
  __syncthreads();
  // thread e -> (column c, row m) with m fastest; stacked row i sits in fragment i/16, register (i%16)%4 of
  // lane ((i%16)/4)*16 + j
  for (int e = threadIdx.x; e < M * 16 * NT; e += THREADS) {
    const int m = e % M, c = e / M;
    const int t = c >> 4, j = c & 15;
    const int i1 = m, i2 = M + m;
    const int a1 = s_acc[i1 >> 4][t][i1 & 3][((i1 & 15) >> 2) * 16 + j];
    const int a2 = s_acc[i2 >> 4][t][i2 & 3][((i2 & 15) >> 2) * 16 + j];
    const int64_t n = n0 + c;
    if (n < N) {
      const float alpha = s_par[m][0];
      const float beta = __fdiv_rn(alpha, a.rg.num2);
      const float ws = e == (int)threadIdx.x ? ws_pre : a.w_scale[n];
      store_out(a.y, a.out_bf16, (int64_t)m * a.ldy + n, merge_scales(ws, alpha, beta, a1, a2));
      if (a.acc1) a.acc1[(int64_t)m * N + n] = a1;
      if (a.acc2) a.acc2[(int64_t)m * N + n] = a2;
    }
  }
}

// ------------------------------------------------------------------ large tiles (prefill)
// v_mfma_i32_32x32x32_i8 (A: row l%32, 16 k bytes of group l/32; D: column l%32, row
// 8*(r/4) + 4*(l/32) + r%4 in register r), BK = 64, LDS double buffering with one barrier per
// K step, global -> register -> LDS staging with the next tile's loads issued before the
// current tile's MFMAs.  LDS rows are 64 B; the 16-byte chunk index is XOR-swizzled with
// (row>>2)&3 so that the ds_read_b128 of sixteen consecutive rows (one 256-byte LDS pass) hit
// sixteen distinct 16-byte bank groups (measured: (row>>1)&3 left a 2-way conflict, half of the
// LDS cycles).
// Each wave owns both components of its activation rows, so the merge stays in registers.
// Workgroup ids are remapped so that each XCD (ids congruent mod 8) walks a contiguous range
// of tiles in groups of kGroupM tile rows: neighbours in an XCD's L2 share W and A tiles.
__device__ __forceinline__ v16i mfma32(v4i a, v4i b, v16i c) {
  return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ v16f mfma32(v4i a, v4i b, v16f c) {  // the 16 bytes are 8 BF16 values
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
}

constexpr int kGroupM = 8;

template <int BMH, int BN, int WM, int WN>
__global__ __launch_bounds__(WM * WN * 64) void gemm_w8_mfma32_kernel(GemmW8Args a, int tiles_m, int tiles_n) {
  constexpr int THREADS = WM * WN * 64;
  constexpr int ROWS_A = 2 * BMH;
  constexpr int TMH = BMH / WM, TN = BN / WN;
  constexpr int FM = TMH / 32, FN = TN / 32;  // fragments per component / per wave column range
  constexpr int LA = ROWS_A * 4 / THREADS, LB = BN * 4 / THREADS;
  static_assert(ROWS_A * 4 % THREADS == 0 && BN * 4 % THREADS == 0, "tile/threads mismatch");
  extern __shared__ __attribute__((aligned(16))) int8_t smem[];
  int8_t* sA = smem;                    // [2][ROWS_A][64]
  int8_t* sB = smem + 2 * ROWS_A * 64;  // [2][BN][64]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int l32 = lane & 31, kg = lane >> 5;
  const int64_t M = a.M, K = a.K, N = a.N;
  // ---- tile of this workgroup (XCD-contiguous, grouped along M)
  const int total = tiles_m * tiles_n;
  int id = blockIdx.x;
  {
    const int per_xcd = (total + 7) / 8;
    const int logical = (id % 8) * per_xcd + id / 8;
    id = logical;
  }
  if (id >= total) return;
  const int group = id / (kGroupM * tiles_n);
  const int first_m = group * kGroupM;
  const int rows_in_group = min(kGroupM, tiles_m - first_m);
  const int in_group = id - group * kGroupM * tiles_n;
  const int tm = first_m + in_group % rows_in_group;
  const int tn = in_group / rows_in_group;
  const int64_t m0 = (int64_t)tm * BMH, n0 = (int64_t)tn * BN;
  const v4i zero4 = {0, 0, 0, 0};

  const int8_t* ga[LA];
  int oa[LA];
  bool va[LA];
#pragma unroll
  for (int i = 0; i < LA; ++i) {
    const int c = tid + i * THREADS, r = c >> 2, ch = c & 3;
    const int comp = r / BMH;
    const int64_t m = m0 + (r - comp * BMH);
    va[i] = m < M;
    ga[i] = (comp ? a.q2 : a.q1) + min(m, M - 1) * a.ldq + ch * 16;
    oa[i] = r * 64 + ((ch ^ ((r >> 2) & 3)) << 4);
  }
  const int8_t* gb[LB];
  int ob[LB];
  bool vb[LB];
#pragma unroll
  for (int i = 0; i < LB; ++i) {
    const int c = tid + i * THREADS, r = c >> 2, ch = c & 3;
    const int64_t n = n0 + r;
    vb[i] = n < N;
    gb[i] = a.W + min(n, N - 1) * K + ch * 16;
    ob[i] = r * 64 + ((ch ^ ((r >> 2) & 3)) << 4);
  }
  const int kch = (tid & 3) * 16;  // k offset of this thread's chunks inside a K step
  v4i ra[LA], rb[LB];
  auto gload = [&](int kt) {
    const int64_t k0 = (int64_t)kt * 64;
    const bool kok = k0 + kch < K;
#pragma unroll
    for (int i = 0; i < LA; ++i) ra[i] = (va[i] && kok) ? ldg16(ga[i] + k0) : zero4;
#pragma unroll
    for (int i = 0; i < LB; ++i) rb[i] = (vb[i] && kok) ? ldg16(gb[i] + k0) : zero4;
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < LA; ++i) *reinterpret_cast<v4i*>(sA + buf * ROWS_A * 64 + oa[i]) = ra[i];
#pragma unroll
    for (int i = 0; i < LB; ++i) *reinterpret_cast<v4i*>(sB + buf * BN * 64 + ob[i]) = rb[i];
  };

  v16i acc[2][FM][FN];
#pragma unroll
  for (int c = 0; c < 2; ++c)
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[c][i][j][r] = 0;

  // fragment addresses inside a buffer (row part; the chunk part depends on the K half-step)
  int fa_row[2][FM], fb_row[FN];
#pragma unroll
  for (int c = 0; c < 2; ++c)
#pragma unroll
    for (int i = 0; i < FM; ++i) fa_row[c][i] = c * BMH + wm * TMH + 32 * i + l32;
#pragma unroll
  for (int j = 0; j < FN; ++j) fb_row[j] = wn * TN + 32 * j + l32;

  const int KT = (int)((K + 63) / 64);
  if (KT > 0) {
    gload(0);
    sstore(0);
  }
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < KT) gload(kt + 1);
    const int8_t* bA = sA + buf * ROWS_A * 64;
    const int8_t* bB = sB + buf * BN * 64;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const int chunk = 2 * s + kg;
      v4i fb[FN];
#pragma unroll
      for (int j = 0; j < FN; ++j)
        fb[j] = *reinterpret_cast<const v4i*>(bB + fb_row[j] * 64 + ((chunk ^ ((fb_row[j] >> 2) & 3)) << 4));
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int i = 0; i < FM; ++i) {
          const v4i fa =
              *reinterpret_cast<const v4i*>(bA + fa_row[c][i] * 64 + ((chunk ^ ((fa_row[c][i] >> 2) & 3)) << 4));
#pragma unroll
          for (int j = 0; j < FN; ++j) acc[c][i][j] = mfma32(fa, fb[j], acc[c][i][j]);
        }
    }
    if (kt + 1 < KT) sstore(buf ^ 1);
    __syncthreads();
  }

  // ---- dual-scale epilogue
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int64_t m = m0 + wm * TMH + 32 * i + (r >> 2) * 8 + kg * 4 + (r & 3);
      if (m >= M) continue;
      const float alpha = a.alpha[m];
      const float beta = __fdiv_rn(alpha, a.rg.num2);
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        const int64_t n = n0 + wn * TN + 32 * j + l32;
        if (n >= N) continue;
        const int a1 = acc[0][i][j][r], a2 = acc[1][i][j][r];
        store_out(a.y, a.out_bf16, m * a.ldy + n, merge_scales(a.w_scale[n], alpha, beta, a1, a2));
        if (a.acc1) a.acc1[m * N + n] = a1;
        if (a.acc2) a.acc2[m * N + n] = a2;
      }
    }
}

// ------------------------------------------------------------------ asynchronous LDS fill (prefill and batched decode)
// Same fragment layout as gemm_w8_mfma32_kernel, but the tiles go HBM/L2 -> LDS with
// global_load_lds_dwordx4 (no staging registers, no ds_write), NS stages deep: while the MFMAs
// of K step t run, the loads of steps t+1 .. t+NS-2 are in flight and step t+NS-1 is being
// issued.  One s_barrier per K step; the wait before it is an explicit s_waitcnt vmcnt(n): a
// wave issues L loads per step and they complete in order.  The loads are written as inline asm
// on purpose: the compiler does not see them write LDS and therefore does not serialise every
// ds_read behind the youngest load.  Each load instruction fills 1 KB of LDS = 16 rows of 64 B in
// lane order, so a lane fetches the global chunk whose swizzled position it owns.  Rows past M / N
// are clamped to the last valid row (their results are never stored).  Requires K % 64 == 0.
//
// Two uses.  <128,256,4,4,4>: prefill, 256x256 output tile (128 activation rows x 2 components)
// on sixteen waves.  Small tiles with many stages: batched decode (32 < M <= 128, few output tiles),
// where the weight stream is cold and the bytes in flight per CU, i.e. the stage count, set the
// HBM rate (Little's law), not the MFMA.
__device__ __forceinline__ void lds_dma16(const int8_t* gbase, uint32_t voff, uint32_t lds_addr) {
  // the base is wave-uniform by construction; say so, or the "s" operand may be given a VGPR pair
  const uint64_t g = reinterpret_cast<uint64_t>(gbase);
  const uint32_t glo = __builtin_amdgcn_readfirstlane((uint32_t)g), ghi = __builtin_amdgcn_readfirstlane((uint32_t)(g >> 32));
  gbase = reinterpret_cast<const int8_t*>(((uint64_t)ghi << 32) | glo);
  lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(voff), "s"(gbase), "s"(lds_addr)
               : "memory", "m0");
}

// Moves one accumulator register to a vector register at this point of the program.  Left to the
// register allocator, an epilogue over 256 accumulators copies all of them out up front, spills, and
// every reload of a spilled value then waits for the stores issued before it.
__device__ __forceinline__ int acc_read(int v) {
  int r;
  asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(r) : "a"(v));
  return r;
}
__device__ __forceinline__ float acc_read(float v) {
  float r;
  asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(r) : "a"(v));
  return r;
}

template <int N>
__device__ __forceinline__ void wait_vm_barrier() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

//
// BF16 = true turns the same pipeline into a plain BF16 GEMM for the comparison path (weights
// already lifted to BF16 in HBM): a 64-byte row chunk is 32 BF16 values instead of 64 codes, the
// matrix instruction is v_mfma_f32_32x32x16_bf16 (same 16 bytes per lane and K group, so the LDS
// layout and every fragment offset are unchanged), the A rows are 2*BMH consecutive activation
// rows instead of two components of BMH rows, and the epilogue stores the fp32 sums.  The
// argument struct is reused with byte units: q1 = activations, ldq and K in bytes, W = BF16 weights.
//
// PROBE = true is a measurement aid (msd_probe_mfma_w8a16): after the first K step the kernel stops
// fetching and keeps multiplying the fragments of that step, i.e. the same MFMA sequence, tile
// schedule and epilogue with real operand bits but no fill, no barrier and no LDS traffic.  Its
// time is what the matrix pipe alone allows for this shape and data on the chip at hand.
//
// KS > 1 (batched decode, where the fill rate of a CU grows with the number of waves that issue loads and the
// tiles are too small to employ many waves): KS groups of WM x WN waves share the tile; every wave takes part
// in the fill, group g multiplies the K extents h = g (mod KS) of every stage, and the groups' integer
// partial sums meet in LDS before the epilogue, whose rows are dealt out over the groups.
template <int BMH, int BN, int WM, int WN, int NS, bool BF16, bool PROBE = false, int BK = 64, int KS = 1>
__global__ __launch_bounds__(WM * WN * KS * 64, (2 * BMH * BN <= 128 * 256 && WM * WN * KS == 4) ? 2 : 1) void gemm_w8_dma_kernel(GemmW8Args a, int tiles_m, int tiles_n) {
  // BK = bytes of K per row and stage.  64: LDS rows of 64 B, chunk swizzle (row>>2)&3, a fill
  // instruction covers 16 rows.  128 (small batched-decode tiles, K % 128 == 0): rows of 128 B =
  // whole cache lines, swizzle (row>>1)&7, 8 rows per fill instruction, four MFMA K extents per
  // stage -- half as many barrier rounds for the same K, which is what bounds those tiles.
  using AccT = std::conditional_t<BF16, v16f, v16i>;
  constexpr int NWT = WM * WN;      // waves that tile the output
  constexpr int NW = NWT * KS, ROWS_A = 2 * BMH, R = ROWS_A + BN;
  constexpr int TMH = BMH / WM, TN = BN / WN, FM = TMH / 32, FN = TN / 32;
  constexpr int HS = BK / 32 / KS;  // MFMA K extents (32 bytes) per stage and wave
  constexpr int CPR = BK / 16;      // 16-byte chunks per row
  constexpr int RPI = 1024 / BK;    // rows per fill instruction
  constexpr int L = R / (RPI * NW);  // fill instructions per wave and stage
  constexpr int STAGE = R * BK;
  static_assert(BK == 64 || BK == 128, "stage depth");
  static_assert(R % (RPI * NW) == 0 && TMH % 32 == 0 && TN % 32 == 0 && BMH % RPI == 0, "tile shape");
  static_assert(NS >= 3 && (NS - 2) * L < 64, "stage count");
  static_assert((BK / 32) % KS == 0 && (KS == 1 || (!BF16 && !PROBE && 16 % KS == 0)), "K groups");
  extern __shared__ __attribute__((aligned(16))) int8_t smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kgrp = wave / NWT, wsub = wave % NWT;
  const int wm = wsub / WN, wn = wsub % WN;
  const int l32 = lane & 31, kg = lane >> 5;
  const int64_t M = a.M, K = a.K, N = a.N;
  const int total = tiles_m * tiles_n;
  int id = blockIdx.x;
  {
    const int per_xcd = (total + 7) / 8;
    id = (id % 8) * per_xcd + id / 8;
  }
  if (id >= total) return;
  const int group = id / (kGroupM * tiles_n);
  const int first_m = group * kGroupM;
  const int rows_in_group = min(kGroupM, tiles_m - first_m);
  const int in_group = id - group * kGroupM * tiles_n;
  const int tm = first_m + in_group % rows_in_group;
  const int tn = in_group / rows_in_group;
  const int64_t m0 = (int64_t)tm * (BF16 ? ROWS_A : BMH), n0 = (int64_t)tn * BN;
  auto swz = [](int row) { return BK == 64 ? ((row >> 2) & 3) : ((row >> 1) & 7); };

  // ---- this wave's L fill instructions per stage: block q*NW + wave of RPI rows
  // (blocks 0 .. ROWS_A/RPI-1 are q1 then q2 rows, the rest W rows)
  const int rr = lane / CPR, pc = lane % CPR;
  uint32_t voff[L];
  const int8_t* gbase[L];
  uint32_t ldst[L];
  const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
  // Blocked activation codes (a.a_step != 0, see GemmW8Args): the block of a stage is one
  // contiguous, already swizzled kilobyte, copied in lane order; a.a_step bytes separate stages.
  const bool blocked = !BF16 && a.a_step != 0;
  int64_t kadv[L];  // bytes between consecutive stages of this instruction's source
#pragma unroll
  for (int q = 0; q < L; ++q) {
    const int blk = q * NW + wave;
    const int lc = pc ^ swz(blk * RPI + rr);  // logical chunk this lane fetches
    kadv[q] = BK;
    if (blk < ROWS_A / RPI) {
      const int comp = blk / (BMH / RPI);
      if (blocked) {
        voff[q] = (uint32_t)(lane * 16);
        gbase[q] = (comp ? a.q2 : a.q1) + (m0 / RPI + blk % (BMH / RPI)) * 1024;
        kadv[q] = a.a_step;
      } else {
        const int64_t mrow = min(m0 + (BF16 ? comp * BMH : 0) + (blk % (BMH / RPI)) * RPI + rr, M - 1);
        voff[q] = (uint32_t)((mrow - m0) * a.ldq + lc * 16);
        gbase[q] = ((comp && !BF16) ? a.q2 : a.q1) + m0 * a.ldq;
      }
    } else if (!BF16 && a.w_packed) {
      // packed weights: the stage's weight region is (BK/64) K steps x (BN/16) channel tiles of one kilobyte,
      // each copied verbatim (lane order); block wb = kk * (BN/16) + nb
      const int wb = blk - ROWS_A / RPI, kk = wb / (BN / 16), nb = wb % (BN / 16);
      const int64_t wtiles = (N + 15) / 16;
      voff[q] = (uint32_t)(lane * 16);
      gbase[q] = a.W + ((int64_t)kk * wtiles + min(n0 / 16 + nb, wtiles - 1)) * 1024;
      kadv[q] = (int64_t)(BK / 64) * wtiles * 1024;
    } else {
      const int64_t nrow = min(n0 + (blk - ROWS_A / RPI) * RPI + rr, N - 1);
      voff[q] = (uint32_t)((nrow - n0) * K + lc * 16);
      gbase[q] = a.W + n0 * K;
    }
    ldst[q] = lds0 + blk * 1024;
  }
  const int KT = (int)(K / BK);
  // Tiles are issued in increasing order, each once: the source of instruction q is a running wave-uniform
  // pointer that advances by its stride after every issue.
  auto uniform64 = [](uint64_t v) {
    // (the builtin returns int: without the casts a low word with bit 31 set would sign-extend over the high word)
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return ((uint64_t)hi << 32) | lo;
  };
#pragma unroll
  for (int q = 0; q < L; ++q) {
    gbase[q] = reinterpret_cast<const int8_t*>(uniform64(reinterpret_cast<uint64_t>(gbase[q])));
    kadv[q] = (int64_t)uniform64((uint64_t)kadv[q]);
  }
  auto issue_one = [&](int kt, int q) {  // q is a compile-time constant at every call site
    lds_dma16(gbase[q], voff[q], ldst[q] + (uint32_t)((kt % NS) * STAGE));
    gbase[q] += kadv[q];
  };
  auto issue = [&](int kt) {
#pragma unroll
    for (int q = 0; q < L; ++q) issue_one(kt, q);
  };

  AccT acc[2][FM][FN];
#pragma unroll
  for (int c = 0; c < 2; ++c)
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[c][i][j][r] = 0;

  int fa_off[2][FM][HS], fb_off[FN][HS];  // byte offset inside a stage for this wave's K extent number hh
#pragma unroll
  for (int hh = 0; hh < HS; ++hh) {
    const int h = hh * KS + kgrp;  // extent of the stage
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int i = 0; i < FM; ++i) {
        const int row = c * BMH + wm * TMH + 32 * i + l32;
        fa_off[c][i][hh] = row * BK + (((2 * h + kg) ^ swz(row)) << 4);
      }
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      const int row = wn * TN + 32 * j + l32;
      if (!BF16 && a.w_packed)  // kilobyte (K step h/2, tile row/16), inside it byte group 2*(h%2)+kg, channel row%16
        fb_off[j][hh] = ROWS_A * BK + (((h >> 1) * (BN / 16) + (row >> 4)) << 10) + (((2 * (h & 1) + kg) * 16 + (row & 15)) << 4);
      else
        fb_off[j][hh] = ROWS_A * BK + row * BK + (((2 * h + kg) ^ swz(row)) << 4);
    }
  }

  auto stage_ptr = [&](int kt) { return smem + (kt % NS) * STAGE; };
  auto load_frags = [&](const int8_t* st, int h, v4i (&fa)[2 * FM], v4i (&fb)[FN]) {
#pragma unroll
    for (int j = 0; j < FN; ++j) fb[j] = *reinterpret_cast<const v4i*>(st + fb_off[j][h]);
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int i = 0; i < FM; ++i) fa[c * FM + i] = *reinterpret_cast<const v4i*>(st + fa_off[c][i][h]);
  };
  auto mfma_block = [&](const v4i (&fa)[2 * FM], const v4i (&fb)[FN]) {
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[c][i][j] = mfma32(fa[c * FM + i], fb[j], acc[c][i][j]);
  };
  // Wait until tile t has landed, then barrier.  In steady state the NS-3 tiles issued after it
  // may stay outstanding ((NS-2) before the first tile); near the end of K fewer tiles follow and
  // the wait simply drains everything.
  auto wait_tile = [&](int t, int newest_issued) {
    const int younger = newest_issued - t;
    if (younger == NS - 2) wait_vm_barrier<(NS - 2) * L>();
    else if (younger == NS - 3) wait_vm_barrier<(NS - 3) * L>();
    else wait_vm_barrier<0>();
  };
  // The first MFMA of a block is issued before the fragment reads of the next block: the
  // compiler's wait for the current fragments (it cannot count LDS operations across the inline
  // asm and waits for all of them) then covers no read that was only just issued.
  auto mfma_first = [&](const v4i (&fa)[2 * FM], const v4i (&fb)[FN]) {
    acc[0][0][0] = mfma32(fa[0], fb[0], acc[0][0][0]);
  };
  auto mfma_rest = [&](const v4i (&fa)[2 * FM], const v4i (&fb)[FN]) {
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          if (c + i + j > 0) acc[c][i][j] = mfma32(fa[c * FM + i], fb[j], acc[c][i][j]);
  };
  // The same block with the L fill instructions of tile kt_issue spread between the MFMAs
  // (one every SPREAD MFMAs): issued in one burst right after the barrier they fill the address
  // queue, the waves leave the burst at different times and the next barrier pays for the skew.
  auto mfma_rest_issue = [&](const v4i (&fa)[2 * FM], const v4i (&fb)[FN], int kt_issue, bool do_issue) {
    constexpr int NM = 2 * FM * FN - 1;
    constexpr int SPREAD = (NM + 1) / L > 1 ? (NM + 1) / L : 1;
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
          const int idx = (c * FM + i) * FN + j - 1;  // 0 .. NM-1 over the MFMAs of this block
          if (idx < 0) continue;
          acc[c][i][j] = mfma32(fa[c * FM + i], fb[j], acc[c][i][j]);
          if (idx % SPREAD == 0 && idx / SPREAD < L) {
            __builtin_amdgcn_sched_barrier(0);
            if (do_issue) issue_one(kt_issue, idx / SPREAD);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
#pragma unroll
    for (int q = (NM + SPREAD - 1) / SPREAD; q < L; ++q)  // loads that found no MFMA to follow
      if (do_issue) issue_one(kt_issue, q);
  };

  // Software pipeline over the K extents (kt, h): the fragments of the next extent are fetched
  // under the MFMAs of the current one, alternating between two register sets.  The barrier for
  // tile kt+1 sits before the last extent of tile kt; after it the stage of tile kt-1 is free and
  // is refilled (tile kt+NS-1) under that extent's MFMAs.
#pragma unroll
  for (int t = 0; t < NS - 1; ++t)
    if (t < KT) issue(t);
  v4i fa0[2 * FM], fb0[FN], fa1[2 * FM], fb1[FN];
  if constexpr (KS > 1) {
    // K groups: few MFMAs per wave and stage and two waves per SIMD, so no fragment pipeline -- wait for the
    // tile, refill the stage every wave has left (all of them passed this barrier after their reads of it),
    // multiply this group's extents.
    for (int kt = 0; kt < KT; ++kt) {
      wait_tile(kt, min(KT - 1, kt + NS - 2));
      if (kt + NS - 1 < KT) issue(kt + NS - 1);
#pragma unroll
      for (int hh = 0; hh < HS; ++hh) {
        load_frags(stage_ptr(kt), hh, fa0, fb0);
        mfma_block(fa0, fb0);
      }
    }
  } else {
  if (KT > 0) {
    wait_tile(0, min(KT - 1, NS - 2));
    load_frags(stage_ptr(0), 0, fa0, fb0);
  }
  // One K stage.  STEADY (a compile-time tag): another tile follows, a tile is issued and the tiles in flight
  // are at their steady count, so the stage is straight-line code; the last NS-1 stages take the general form.
  auto stage = [&](int kt, auto steady_tag) {
    constexpr bool STEADY = decltype(steady_tag)::value;
    if constexpr (PROBE) {
      if (kt > 0) {
#pragma unroll
        for (int h = 0; h < HS; h += 2) {
          mfma_block(fa0, fb0);
          __builtin_amdgcn_sched_barrier(0);
          mfma_block(fa1, fb1);
          __builtin_amdgcn_sched_barrier(0);
        }
        return;
      }
    }
    const bool more = STEADY || kt + 1 < KT;
#pragma unroll
    for (int h = 0; h < HS; ++h) {
      const bool last = h == HS - 1;
      v4i(&fac)[2 * FM] = (h & 1) ? fa1 : fa0;
      v4i(&fbc)[FN] = (h & 1) ? fb1 : fb0;
      v4i(&fan)[2 * FM] = (h & 1) ? fa0 : fa1;
      v4i(&fbn)[FN] = (h & 1) ? fb0 : fb1;
      if (last && more) {
        if constexpr (STEADY) wait_vm_barrier<(NS - 3) * L>();
        else wait_tile(kt + 1, min(KT - 1, kt + NS - 2));
      }
      mfma_first(fac, fbc);
      __builtin_amdgcn_sched_barrier(0);
      if (!last) load_frags(stage_ptr(kt), h + 1, fan, fbn);
      else if (more) load_frags(stage_ptr(kt + 1), 0, fan, fbn);
      __builtin_amdgcn_sched_barrier(0);
      if (last) mfma_rest_issue(fac, fbc, kt + NS - 1, STEADY || (!PROBE && more && kt + NS - 1 < KT));
      else mfma_rest(fac, fbc);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  int kt = 0;
  if constexpr (!PROBE)
    for (; kt + NS - 1 < KT; ++kt) stage(kt, std::true_type{});
  for (; kt < KT; ++kt) stage(kt, std::false_type{});
  }

  if constexpr (BF16) {
    // ---- plain epilogue of the comparison GEMM
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int64_t m = m0 + c * BMH + wm * TMH + 32 * i + (r >> 2) * 8 + kg * 4 + (r & 3);
          if (m < M) {
#pragma unroll
            for (int j = 0; j < FN; ++j) {
              const int64_t n = n0 + wn * TN + 32 * j + l32;
              if (n < N) store_out_stream(a.y, a.out_bf16, m * a.ldy + n, acc_read(acc[c][i][j][r]));
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
    return;
  } else {
  // ---- dual-scale epilogue.  alpha and beta of the tile's rows go through LDS (free now), the
  // output is produced one (fragment, register) row at a time so that the compiler does not pull
  // all accumulators into VGPRs at once.
  __syncthreads();
  constexpr int NACC = 2 * FM * FN * 16;                  // accumulator registers per lane
  constexpr int RED_BYTES = KS > 1 ? NW * NACC * 256 : 0;  // K groups: every wave's partial sums, [wave][register][lane]
  int* red = reinterpret_cast<int*>(smem);
  if constexpr (KS > 1) {
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            red[(wave * NACC + ((c * FM + i) * FN + j) * 16 + r) * 64 + lane] = acc[c][i][j][r];
  }
  float* s_ab = reinterpret_cast<float*>(smem + RED_BYTES);  // [0..BMH-1] alpha, [BMH..2BMH-1] beta
  for (int i = tid; i < BMH; i += NW * 64) {
    const int64_t m = m0 + i;
    const float al = m < M ? a.alpha[m] : 0.f;
    s_ab[i] = al;
    s_ab[BMH + i] = __fdiv_rn(al, a.rg.num2);
  }
  __syncthreads();
  // The weight scales are fetched unconditionally (clamped column) and pinned in registers before the
  // store loops: a load still pending inside the conditional store code makes the compiler wait for
  // ALL vector-memory operations before each use, i.e. for the previous store's completion, and the
  // epilogue then runs at one store round trip per row.
  float sw[FN];
#pragma unroll
  for (int j = 0; j < FN; ++j) sw[j] = a.w_scale[min(n0 + wn * TN + 32 * j + l32, N - 1)];
#pragma unroll
  for (int j = 0; j < FN; ++j) asm volatile("" : "+v"(sw[j]));
  // one pass per kind of output, each under a single uniform branch
  auto for_rows = [&](auto&& emit) {
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if (KS > 1 && r % KS != kgrp) continue;  // this row belongs to another K group (wave-uniform)
        const int lr = wm * TMH + 32 * i + (r >> 2) * 8 + kg * 4 + (r & 3);
        const int64_t m = m0 + lr;
        const float alpha = s_ab[lr], beta = s_ab[BMH + lr];
        if (m < M) {
#pragma unroll
          for (int j = 0; j < FN; ++j) {
            const int64_t n = n0 + wn * TN + 32 * j + l32;
            if (n >= N) continue;
            if constexpr (KS > 1) {
              int a1 = 0, a2 = 0;
#pragma unroll
              for (int g = 0; g < KS; ++g) {
                const int* rw = red + (((g * NWT + wsub) * NACC + (i * FN + j) * 16 + r) * 64 + lane);
                a1 += rw[0];
                a2 += rw[FM * FN * 16 * 64];
              }
              emit(m, n, sw[j], alpha, beta, a1, a2);
            } else {
              emit(m, n, sw[j], alpha, beta, acc_read(acc[0][i][j][r]), acc_read(acc[1][i][j][r]));
            }
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
  };
  if (a.out_bf16) {
    uint16_t* y = reinterpret_cast<uint16_t*>(a.y);
    for_rows([&](int64_t m, int64_t n, float s, float alpha, float beta, int a1, int a2) {
      __builtin_nontemporal_store(f32_to_bf16_bits(merge_scales(s, alpha, beta, a1, a2)), y + m * a.ldy + n);
    });
  } else {
    float* y = reinterpret_cast<float*>(a.y);
    for_rows([&](int64_t m, int64_t n, float s, float alpha, float beta, int a1, int a2) {
      __builtin_nontemporal_store(merge_scales(s, alpha, beta, a1, a2), y + m * a.ldy + n);
    });
  }
  if (a.acc1 || a.acc2) {  // observation points for the parity tests
    for_rows([&](int64_t m, int64_t n, float, float, float, int a1, int a2) {
      if (a.acc1) a.acc1[m * N + n] = a1;
      if (a.acc2) a.acc2[m * N + n] = a2;
    });
  }
  }
}

template <int BMH, int BN, int WM, int WN, int NS, bool BF16 = false, bool PROBE = false, int BK = 64, int KS = 1>
static int launch_dma(const GemmW8Args& a, hipStream_t stream) {
  if (a.K % BK != 0 || (a.a_step != 0 && a.a_bk != BK)) return MSD_ERR_INVALID_ARG;
  const int tiles_m = (int)cdiv(a.M, BF16 ? 2 * BMH : BMH), tiles_n = (int)cdiv(a.N, BN);
  const int total = tiles_m * tiles_n;
  const int grid = ((total + 7) / 8) * 8;
  // the stages; with K groups the partial sums of all waves (256 B per accumulator register) plus the row scales
  constexpr size_t kStages = (size_t)NS * (2 * BMH + BN) * BK;
  constexpr size_t kReduce = KS > 1 ? (size_t)WM * WN * KS * (2 * (BMH / WM / 32) * (BN / WN / 32) * 16) * 256 + 2 * BMH * 4 : 0;
  constexpr size_t lds = kStages > kReduce ? kStages : kReduce;
  static_assert(lds <= 160 * 1024, "LDS budget");
  static bool attr_set = false;
  if (!attr_set) {
    MSD_HIP_CHECK(hipFuncSetAttribute(
        reinterpret_cast<const void*>(&gemm_w8_dma_kernel<BMH, BN, WM, WN, NS, BF16, PROBE, BK, KS>),
        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_set = true;
  }
  hipLaunchKernelGGL((gemm_w8_dma_kernel<BMH, BN, WM, WN, NS, BF16, PROBE, BK, KS>), dim3(grid), dim3(WM * WN * KS * 64),
                     lds, stream, a, tiles_m, tiles_n);
  return MSD_OK;
}

template <int BMH, int BN, int WM, int WN>
static int launch_mfma32(const GemmW8Args& a, hipStream_t stream) {
  const int tiles_m = (int)cdiv(a.M, BMH), tiles_n = (int)cdiv(a.N, BN);
  const int total = tiles_m * tiles_n;
  const int grid = ((total + 7) / 8) * 8;  // every XCD gets the same number of slots
  const size_t lds = (size_t)2 * (2 * BMH + BN) * 64;
  static bool attr_set = false;
  if (!attr_set && lds > 64 * 1024) {
    MSD_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_w8_mfma32_kernel<BMH, BN, WM, WN>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_set = true;
  }
  hipLaunchKernelGGL((gemm_w8_mfma32_kernel<BMH, BN, WM, WN>), dim3(grid), dim3(WM * WN * 64), lds, stream, a,
                     tiles_m, tiles_n);
  return MSD_OK;
}

// Plain BF16 GEMM y = x Wb^T (fp32 accumulation) on the asynchronous-fill pipeline, for the
// comparison path.  x [M][ldx] BF16 (rows 16-byte aligned), Wb [N][K] BF16, K % 32 == 0.
int launch_bf16_gemm_tiled(const uint16_t* x, int64_t M, int64_t K, int64_t ldx, const uint16_t* Wb, int64_t N,
                           void* y, int out_bf16, int64_t ldy, hipStream_t stream) {
  GemmW8Args a{};
  a.q1 = reinterpret_cast<const int8_t*>(x);
  a.q2 = a.q1;
  a.ldq = 2 * ldx;
  a.W = reinterpret_cast<const int8_t*>(Wb);
  a.y = y;
  a.out_bf16 = out_bf16;
  a.ldy = ldy;
  a.M = M;
  a.K = 2 * K;
  a.N = N;
  const int rc = launch_dma<128, 256, 4, 4, 4, true>(a, stream);
  if (rc) return rc;
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

// ------------------------------------------------------------------ one-time weight packing
// W [N][K] (K % 64 == 0) -> Wp[K/64][ceil(N/16)][1 KB] (GemmW8Args::w_packed).  One thread per 16 bytes.
__global__ __launch_bounds__(256) void pack_weights_w8_kernel(const int8_t* __restrict__ W, int64_t N, int64_t K,
                                                              int8_t* __restrict__ P) {
  const int64_t tiles = (N + 15) / 16;
  const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;  // 16-byte piece of the packed array
  if (id >= (K / 64) * tiles * 64) return;
  const int l = (int)(id & 63);
  const int64_t blk = id >> 6, ks = blk / tiles, nb = blk % tiles;
  const int64_t n = nb * 16 + (l & 15);
  v4i v = {0, 0, 0, 0};
  if (n < N) v = ldg16(W + n * K + ks * 64 + 16 * (l >> 4));
  *reinterpret_cast<v4i*>(P + id * 16) = v;
}

int launch_pack_weights_w8(const int8_t* W, int64_t N, int64_t K, int8_t* packed, hipStream_t stream) {
  const int64_t pieces = (K / 64) * ((N + 15) / 16) * 64;
  if (pieces == 0) return MSD_OK;
  hipLaunchKernelGGL(pack_weights_w8_kernel, dim3((unsigned)cdiv(pieces, 256)), dim3(256), 0, stream, W, N, K, packed);
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

// ------------------------------------------------------------------ dispatch
// Which instance of the everything-in-flight single-launch kernel serves (K, N): 0 = none.
//   K = 1024 / 2048 / 4096 / 8192 as 4 x 4, 4 x 8, 4 x 16 (or 8 x 8), 8 x 16 (waves x K steps per wave); with many
//   column tiles two or four tiles per workgroup.
enum { kFusedNone = 0, kFused4x4, kFused4x8, kFused4x16, kFused4x16x2, kFused8x8x4, kFused8x16, kFused8x16x2 };
static int fused_instance(int64_t M, int64_t K, int64_t N) {
  const bool wide = cdiv(N, 16) > 512;
  // (Twice as many elements measured slower inside a graph, where a dependent launch costs 2 us: 10.3 against 9.5 us
  // at 8 x 4096 x 4096 -- and faster when every launch also costs host time, which is not what is timed here.)
  if (M < 1 || M > kFusedMaxRows || M * K > kFusedMaxElems) return kFusedNone;
  if (K == 1024) return kFused4x4;
  if (K == 2048) return kFused4x8;
  if (K == 4096) return !wide ? kFused4x16 : M <= 2 ? kFused4x16x2 : kFused8x8x4;
  if (K == 8192) return wide ? kFused8x16x2 : kFused8x16;
  return kFusedNone;
}

// Single launch (the GEMM kernel decomposes the activations itself)?  The general form (any K) pays beyond two
// rows more for the repeated decomposition than for a launch (measured); the everything-in-flight form up to
// kFusedMaxElems activation elements.
bool gemm_w8_is_fused(int64_t M, int64_t K, int64_t N) {
  if (fused_instance(M, K, N) != kFusedNone) return true;
  return M <= 2 && K > 0 && 2 * M * (K + 1024) <= kSelfMaxCodeBytes;
}

template <int WAVES, int STEPS, int NT, int MR>
static int launch_fused_mr(const GemmW8Args& a, hipStream_t stream) {
  const dim3 grid((unsigned)cdiv(a.N, 16 * NT));
  const size_t dyn = (size_t)WAVES * 2 * a.M * (STEPS * 64 + 16);
  static bool attr_set = false;  // per instantiation
  if (!attr_set) {
    MSD_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_w8_fused_kernel<WAVES, STEPS, NT, MR>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSelfMaxCodeBytes));
    MSD_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_w8_fused_kernel<WAVES, STEPS, NT, MR, true>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)(kSelfMaxCodeBytes - WAVES * 4096)));
    attr_set = true;
  }
  // canonical weights and many column tiles: row-segment loads (4096 x 14336, one row: 14.2 -> 12.7 us; with few
  // tiles the call is latency-bound and the trip through LDS shows: 5.75 -> 6.0 us at 4096 x 4096)
  if (!a.w_packed && cdiv(a.N, 16) > 512)
    hipLaunchKernelGGL((gemm_w8_fused_kernel<WAVES, STEPS, NT, MR, true>), grid, dim3(WAVES * 64), dyn, stream, a);
  else
    hipLaunchKernelGGL((gemm_w8_fused_kernel<WAVES, STEPS, NT, MR>), grid, dim3(WAVES * 64), dyn, stream, a);
  return MSD_OK;
}

// picks the row bound: M * K <= kFusedMaxElems, at most four 16-element chunks of x per lane
template <int WAVES, int STEPS, int NT>
static int launch_fused(const GemmW8Args& a, hipStream_t stream) {
  constexpr int kByElems = (int)(kFusedMaxElems / (WAVES * STEPS * 64)), kByChunks = 64 / STEPS;  // XC <= 4
  constexpr int MAXR = kByElems < kByChunks ? (kByElems < kFusedMaxRows ? kByElems : kFusedMaxRows)
                                            : (kByChunks < kFusedMaxRows ? kByChunks : kFusedMaxRows);
  if (a.K != (int64_t)WAVES * STEPS * 64 || a.M > MAXR) return MSD_ERR_INVALID_ARG;
  if (a.M <= 1) return launch_fused_mr<WAVES, STEPS, NT, 1>(a, stream);
  if (a.M <= 2) return launch_fused_mr<WAVES, STEPS, NT, 2>(a, stream);
  if constexpr (MAXR >= 4) {
    if (a.M <= 4) return launch_fused_mr<WAVES, STEPS, NT, 4>(a, stream);
  }
  if constexpr (MAXR >= 8) {
    if (a.M <= 8) return launch_fused_mr<WAVES, STEPS, NT, 8>(a, stream);
  }
  return MSD_ERR_INVALID_ARG;
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
          reinterpret_cast<const void*>(&gemm_w8_decode_kernel<WAVES, UNROLL, RT, NT, SELF, true>),
          hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSelfMaxCodeBytes));
      MSD_HIP_CHECK(hipFuncSetAttribute(
          reinterpret_cast<const void*>(&gemm_w8_decode_kernel<WAVES, UNROLL, RT, NT, SELF, false>),
          hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSelfMaxCodeBytes));
      allowed = kSelfMaxCodeBytes;
    }
  }
  if constexpr (!SELF && UNROLL % 4 == 0) {
    // canonical weights, every wave's K range a whole number of 256-byte row segments
    if (!a.w_packed && a.K % (WAVES * 256) == 0) {
      hipLaunchKernelGGL((gemm_w8_decode_kernel<WAVES, UNROLL, RT, NT, false, true, true>), grid, dim3(WAVES * 64), 0, stream, a);
      return MSD_OK;
    }
  }
  if (a.K % 64 == 0)
    hipLaunchKernelGGL((gemm_w8_decode_kernel<WAVES, UNROLL, RT, NT, SELF, true>), grid, dim3(WAVES * 64), dyn, stream, a);
  else
    hipLaunchKernelGGL((gemm_w8_decode_kernel<WAVES, UNROLL, RT, NT, SELF, false>), grid, dim3(WAVES * 64), dyn, stream, a);
  return MSD_OK;
}

template <int WAVES, int UNROLL, int RT, int NT>
static int launch_rowsplit(const GemmW8Args& a, hipStream_t stream) {
  const dim3 grid((unsigned)cdiv(a.N, 16 * NT), (unsigned)cdiv(a.M, 8 * RT));
  if (a.K % 64 == 0)
    hipLaunchKernelGGL((gemm_w8_rowsplit_kernel<WAVES, UNROLL, RT, NT, true>), grid, dim3(WAVES * 64), 0, stream, a);
  else
    hipLaunchKernelGGL((gemm_w8_rowsplit_kernel<WAVES, UNROLL, RT, NT, false>), grid, dim3(WAVES * 64), 0, stream, a);
  return MSD_OK;
}

int launch_gemm_w8_grouped(const GemmW8Args& a, const int32_t* offs, int E, hipStream_t stream) {
  if (E <= 0 || a.N == 0) return MSD_OK;
  constexpr int NT = 2;
  const dim3 grid((unsigned)cdiv(a.N, 16 * NT), (unsigned)E);
  // (canonical weights only; the K range of each of the eight waves a whole number of 256-byte row segments)
  if (a.K % 2048 == 0 && !a.w_packed)
    hipLaunchKernelGGL((gemm_w8_grouped_kernel<8, 4, 2, NT, true, true>), grid, dim3(8 * 64), 0, stream, a, offs);
  else if (a.K % 64 == 0)
    hipLaunchKernelGGL((gemm_w8_grouped_kernel<8, 4, 2, NT, true>), grid, dim3(8 * 64), 0, stream, a, offs);
  else
    hipLaunchKernelGGL((gemm_w8_grouped_kernel<8, 4, 2, NT, false>), grid, dim3(8 * 64), 0, stream, a, offs);
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

// Measurement aid: the prefill kernel's MFMA sequence without its data movement (PROBE above).
int launch_gemm_w8_mfma_probe(const GemmW8Args& a, hipStream_t stream) {
  if (a.M == 0 || a.N == 0) return MSD_OK;
  if (a.K % 64 != 0 || a.K < 64 || a.x != nullptr) return MSD_ERR_SHAPE;
  const int rc = launch_dma<128, 256, 4, 4, 4, false, true>(a, stream);
  if (rc) return rc;
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

// Which kernel family serves a shape (the decomposition launch writes the layout it wants).
enum class W8Path { kDecode, kFillSmall, kFillLarge, kStaged };
static W8Path w8_path(int64_t M, int64_t K, int64_t N) {
  const bool wide = cdiv(N, 16) > 512;  // many column tiles
  const bool k64 = K % 64 == 0 && K >= 64;
  if (2 * M <= 32) return W8Path::kDecode;
  if (2 * M <= 64) return (wide && k64) ? W8Path::kFillSmall : W8Path::kDecode;
  if (cdiv(M, 128) * cdiv(N, 256) < 128) return k64 ? W8Path::kFillSmall : W8Path::kStaged;
  return k64 ? W8Path::kFillLarge : W8Path::kStaged;
}

// Fragments of the fragment-major code layout this shape's GEMM reads (the register-operand kernels); 0: not used.
int gemm_w8_frag_rt(int64_t M, int64_t K, int64_t N) {
  if (gemm_w8_is_fused(M, K, N) || K % 64 != 0 || K < 64) return 0;
  if (w8_path(M, K, N) != W8Path::kDecode) return 0;
  return 2 * M <= 16 ? 1 : 2 * M <= 32 ? 2 : 2 * M <= 48 ? 3 : 4;
}

// Stage depth (bytes of K per row) of the blocked code layout this shape's GEMM reads; 0: row-major.
int gemm_w8_blocked_bk(int64_t M, int64_t K, int64_t N) {
  if (gemm_w8_is_fused(M, K, N)) return 0;
  const W8Path p = w8_path(M, K, N);
  if (p == W8Path::kFillLarge) return 64;
  if (p == W8Path::kFillSmall) return K % 128 == 0 ? 128 : 64;
  return 0;
}

int launch_gemm_w8(const GemmW8Args& a, hipStream_t stream) {
  if (a.M == 0 || a.N == 0) return MSD_OK;
  const int64_t M = a.M, N = a.N;
  int rc = MSD_OK;
  const bool wide = cdiv(N, 16) > 512;  // many column tiles: widen the workgroup tile (measured)
  const W8Path path = w8_path(M, a.K, N);
  if (a.a_step != 0 && (a.x != nullptr || (path != W8Path::kFillSmall && path != W8Path::kFillLarge)))
    return MSD_ERR_INVALID_ARG;  // only the asynchronous-fill kernels read the blocked layout
  if ((a.a_step != 0 || a.x != nullptr) && a.a_frag != 0) return MSD_ERR_INVALID_ARG;
  if (a.x != nullptr) {  // the caller asked for the single-launch path (gemm_w8_is_fused)
    switch (fused_instance(M, a.K, N)) {
      case kFused4x4: rc = launch_fused<4, 4, 1>(a, stream); break;
      case kFused4x8: rc = launch_fused<4, 8, 1>(a, stream); break;
      case kFused4x16: rc = launch_fused<4, 16, 1>(a, stream); break;
      case kFused4x16x2: rc = launch_fused<4, 16, 2>(a, stream); break;
      case kFused8x8x4: rc = launch_fused<8, 8, 4>(a, stream); break;
      case kFused8x16: rc = launch_fused<8, 16, 1>(a, stream); break;
      case kFused8x16x2: rc = launch_fused<8, 16, 2>(a, stream); break;
      default: rc = launch_decode<4, 8, 1, 1, true>(a, stream);
    }
  } else if (a.a_frag != 0) {
    // fragment-major codes (gemm_w8_frag_rt): the register-operand kernel, with the whole K range of a wave in
    // one batch of loads where the registers allow it (measured against the instances below at K = 4096)
    if (path != W8Path::kDecode || a.a_frag != (2 * M <= 16 ? 1 : 2 * M <= 32 ? 2 : 2 * M <= 48 ? 3 : 4)) return MSD_ERR_INVALID_ARG;
    if (a.a_frag == 1)
      rc = wide ? launch_decode<4, 8, 1, 2, false>(a, stream) : launch_decode<4, 16, 1, 1, false>(a, stream);
    else if (a.a_frag == 2)
      rc = wide ? launch_decode<8, 4, 2, 2, false>(a, stream) : launch_decode<4, 16, 2, 1, false>(a, stream);
    else if (a.a_frag == 3)  // 17..24 rows: three fragments instead of four
      rc = wide ? launch_decode<8, 2, 3, 4, false>(a, stream) : launch_decode<8, 8, 3, 1, false>(a, stream);
    else
      // (eight waves x 8 steps: a wave's whole K range at K = 4096 in one batch, 13.35 against 13.6 us at 32 rows;
      // sixteen waves x 4 steps 13.8)
      rc = wide ? launch_decode<8, 2, 4, 4, false>(a, stream) : launch_decode<8, 8, 4, 1, false>(a, stream);
  } else if (path == W8Path::kDecode) {
    if (2 * M <= 16)
      rc = wide ? launch_decode<4, 8, 1, 2, false>(a, stream) : launch_decode<4, 8, 1, 1, false>(a, stream);
    else if (2 * M <= 32)
      rc = launch_decode<8, 4, 2, 2, false>(a, stream);
    else
      rc = wide ? launch_decode<8, 2, 4, 4, false>(a, stream) : launch_rowsplit<8, 4, 2, 2>(a, stream);
  } else if (path == W8Path::kFillSmall) {
    // Few output tiles (decode with a large batch): asynchronous-fill kernel on the largest of three
    // small tiles that still gives about 200 workgroups (measured: the stream rate is set by how
    // many CUs pull, then by the activation re-reads per workgroup).  16 < M <= 32 with many
    // columns measured 27 vs 31 us on the smallest tile against the register-operand kernel.
    // These tiles do few MFMAs per barrier round, so with K % 128 == 0 a stage holds 128 bytes of K.
    const auto wgs = [&](int bmh, int bn) { return cdiv(M, bmh) * cdiv(N, bn); };
    const bool deep = a.K % 128 == 0 && (a.a_step == 0 || a.a_bk == 128);
    // Up to one workgroup per CU of the smallest tile: eight waves as four K groups (measured 16.5 vs 20.5 us at
    // 128 x 4096 x 4096, 19 vs 22 us at 32 x 4096 x 14336; with more tiles than CUs the larger tiles win again).
    // At most half a chip of those: tiles of 32 channels, four waves (the four K groups of one 32 x 32 tile), two
    // workgroups per CU.
    if (deep && wgs(32, 64) <= 128)
      rc = launch_dma<32, 32, 1, 1, 4, false, false, 128, 4>(a, stream);
    else if (deep && wgs(32, 64) <= 256)
      rc = launch_dma<32, 64, 1, 2, 4, false, false, 128, 4>(a, stream);
    else
    // eight waves measured 30 vs 31.6 us at 128 x 4096 x 14336; as 2 x 2 waves in two K groups (a third fewer
    // fragment reads) 31.4, as sixteen waves (2 x 4 in two K groups) 31.3
    if (2 * M > 64 && wgs(64, 128) >= 200)
      rc = deep ? launch_dma<64, 128, 2, 4, 4, false, false, 128>(a, stream) : launch_dma<64, 128, 2, 2, 8>(a, stream);
    else if (2 * M > 64 && wgs(64, 64) >= 200)
      rc = deep ? launch_dma<64, 64, 2, 2, 4, false, false, 128>(a, stream) : launch_dma<64, 64, 2, 2, 6>(a, stream);
    else  // at most 64 KB of LDS: two workgroups per CU
      rc = deep ? launch_dma<32, 64, 1, 2, 4, false, false, 128>(a, stream) : launch_dma<32, 64, 1, 2, 8>(a, stream);
  } else if (path == W8Path::kFillLarge) {
    // Sixteen waves (four per SIMD, 64x64 wave tiles of 64 accumulator registers): 0.5-5 % faster over the four
    // benchmark shapes than eight waves with 128x64 wave tiles (280 against 294 us at 2048 x 8192 x 8192), which in
    // turn measured 6-10 % faster than four waves with 128x128 wave tiles -- more waves issue fill instructions and
    // a SIMD always has another wave to issue from while one waits.  Three or five stages, half-size tiles (two
    // workgroups per CU) and 128 bytes of K per barrier on 64x256 or 128x128 tiles (a 256x256 tile of 128-byte
    // stages does not fit LDS three deep) measured no better.
    rc = launch_dma<128, 256, 4, 4, 4>(a, stream);
  } else if (cdiv(M, 128) * cdiv(N, 256) < 128) {
    rc = launch_mfma32<64, 64, 2, 2>(a, stream);
  } else {
    rc = launch_mfma32<128, 256, 2, 2>(a, stream);
  }
  if (rc) return rc;
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

}  // namespace msd
