// W4A16 MSD GEMM for 5 to 128 activation rows, where the weight stream is the bound (batched
// decode): paper Sec. 3.2.1 / Alg. 2 feeding Sec. 3.4.1 on v_mfma_scale_f32_32x32x64_f8f6f4.
//
// Two launches per call: the K-step-major decomposition of gemm_w4_prefill.hip (per group of 32
// rows 3 KB of FP6 operands per K step of 64 elements, plus one scale record per K step), then this
// kernel.
//
// One workgroup = 4 waves = 128 output channels, the whole K range, all rows (one, two or four
// groups of 32); a wave owns 32 channels (lane l: channel l%32, MX block l/32 of each K step).  (Eight waves in
// two K groups measured no better at 32 rows and worse at 128, where the registers no longer suffice.)  K is
// walked in batches of U steps.  Per batch the workgroup stages the weights (128 channels x U*32
// bytes, contiguous per channel and instruction) and the activation operands of the batch (hot in
// L2, shared by the four waves) through LDS, double-buffered: global -> registers, registers -> LDS
// one batch later (two register stages, so that two batches are in flight while a third is
// multiplied), one barrier per batch.  Weight rows sit in LDS with a 16-byte pad, which makes both
// the staging stores and the fragment reads (32 rows at one K offset) conflict-free.  The weights'
// scale bytes (2U per channel and batch) go straight to registers.  Both components accumulate
// into one fp32 accumulator of 16 registers per row group (scale bytes alpha and alpha - shift).
// Why not weights straight into the B operand, as in the skinny kernel: with the 32 x 32 x 64
// instruction only two lanes share a weight row, so every load instruction touches 32 rows with 32
// bytes each -- measured 55 us (cacheable) to 68 us (non-temporal) at M = 32, N = 28672, K = 8192,
// against 44 us with staging, and against 78 us for the skinny kernel, which re-reads the activation
// operands for every 16 channels.
#include <type_traits>

#include "kernels.hpp"

namespace msd {

namespace {

constexpr int kMidThreads = 256;
constexpr int kMidBN = 128;  // channels per workgroup

// RG: groups of 32 activation rows held at once (M <= 32 * RG); U: K steps per batch (U * 32 weight
// bytes per channel).  Per batch and buffer LDS holds U * (RG * 3072 + 256) bytes of activation
// operands and scale dwords and 128 padded weight rows; (RG, U) = (1, 8), (2, 4), (4, 4) fit twice.
// A4: the components are OCP E2M1 codes (the E2M1-grid ablation) carried as native FP4 operands: 2 KB per
// 32-row group and K step (chunk 2c+b = [32 rows][16 B of block b of component c]) instead of 3 KB.
template <int RG, int U, bool A4>
struct MidCfg {
  static constexpr int kGroupA = A4 ? 2048 : 3072;                         // operand bytes of a 32-row group per K step
  static constexpr int kStepA = RG * kGroupA;                              // operand bytes per K step
  static constexpr int kStageA = U * kStepA / 16 / kMidThreads;            // 16-byte operand chunks per thread and batch
  static constexpr int kChunksW = U * 2;                                   // 16-byte chunks per weight row and batch
  static constexpr int kRowsPerPass = kMidThreads / kChunksW;              // weight rows one staging instruction covers
  static constexpr int kStageW = kMidBN / kRowsPerPass;                    // 16-byte weight chunks per thread and batch
  static constexpr int kRowW = U * 32 + 16;                                // LDS bytes per weight row (padded)
  static constexpr int kBufA = U * (kStepA + 256);                         // operands, then the scale dwords
  static constexpr int kBufW = kMidBN * kRowW;
  static constexpr int kLds = 2 * (kBufA + kBufW);
  static_assert(kStageA * kMidThreads * 16 == U * kStepA && U * 16 <= kMidThreads, "batch split");
  static_assert(kRowsPerPass * kChunksW == kMidThreads && kStageW * kRowsPerPass == kMidBN, "weight staging split");
  static_assert(U % 2 == 0 && U <= 8, "one 16-byte scale load per channel covers at most 16 blocks");
  static_assert(kLds <= 160 * 1024, "LDS budget");
};

template <int SEL, int CBSZ>
__device__ __forceinline__ v16f mfma_mid(v8i a, v8i b, v16f c, int sa, int sb) {
  // A: FP6 E2M3 (cbsz = 2) or FP4 E2M1 (cbsz = 4), B: FP4 E2M1 (blgp = 4); E8M0 scales: byte SEL of sa,
  // byte 0 of sb
  return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, CBSZ, 4, SEL, sa, 0, sb);
}

template <int RG, int U, bool A4>
__global__ __launch_bounds__(kMidThreads) void gemm_w4_mid_kernel(const uint8_t* __restrict__ qop,
                                                                  const uint8_t* __restrict__ sa_t,
                                                                  const uint8_t* __restrict__ W,
                                                                  const uint8_t* __restrict__ We, void* y,
                                                                  int out_bf16, int64_t ldy, int M, int64_t K,
                                                                  int64_t N, int shift, int w_packed) {
  using C = MidCfg<RG, U, A4>;
  constexpr int CBSZ = A4 ? 4 : 2;
  extern __shared__ __attribute__((aligned(16))) uint8_t s_mid[];  // [2][A batch] then [2][W batch]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, kb = lane >> 5;
  const int64_t n0 = (int64_t)blockIdx.x * kMidBN;
  const int64_t n = n0 + wave * 32 + l32;
  // channels past N repeat the last one; their results are not stored
  // Packed weights (msd_pack_weights_w4): W is [K/128][tiles][1 KB], kilobyte = 16 channels x 4 MX blocks in the
  // order (block g, channel r); We is [K/512][tiles][16 channels][16 bytes].
  const int64_t wtiles = (N + 15) / 16;
  const int64_t nc = min(n, N - 1);
  const uint8_t* werow = w_packed ? We + (nc / 16) * 256 + (nc % 16) * 16 : We + nc * (K / 32);
  const int NB = (int)(K / (64 * U));  // batches (K is a multiple of 64 * U)
  // weight staging, canonical layout: chunk tid + i * 256 of the batch = (row chunk / kChunksW, 16-byte column
  // chunk % kChunksW).  Packed layout: pass i of wave w copies kilobyte 4 i + w of the batch's U/2 x 8 kilobytes
  // (K unit (4 i + w) / 8, channel tile (4 i + w) % 8), lane (g, r) to row 16 tile + r, byte 64 unit + 16 g.
  const int wr = tid / C::kChunksW, wc = tid % C::kChunksW;
  const uint8_t* wsrc[C::kStageW];
  int wdst[C::kStageW];
#pragma unroll
  for (int i = 0; i < C::kStageW; ++i) {
    if (w_packed) {
      const int kb_i = 4 * i + wave, unit = kb_i >> 3, tile = kb_i & 7;
      wsrc[i] = W + ((int64_t)unit * wtiles + min(n0 / 16 + tile, wtiles - 1)) * 1024 + lane * 16;
      wdst[i] = (tile * 16 + (lane & 15)) * C::kRowW + unit * 64 + (lane >> 4) * 16;
    } else {
      wsrc[i] = W + min(n0 + wr + C::kRowsPerPass * i, N - 1) * (K / 2) + wc * 16;
      wdst[i] = (wr + C::kRowsPerPass * i) * C::kRowW + wc * 16;
    }
  }
  const int64_t wstep = w_packed ? (int64_t)(U / 2) * wtiles * 1024 : U * 32;  // weight bytes between batches

  // two register stages: while batch b is multiplied out of LDS, batch b + 1 and batch b + 2 are in flight
  struct Stage {
    v4i w[C::kStageW], a[C::kStageA], asc, wsc;  // wsc: the 2 U weight scale bytes of this lane's channel
  };
  Stage st0, st1;
  st0.asc = st1.asc = v4i{0, 0, 0, 0};
  st0.wsc = st1.wsc = v4i{0, 0, 0, 0};
  auto load_batch = [&](int b, Stage& st) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < C::kStageW; ++i)
      st.w[i] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(wsrc[i] + (int64_t)b * wstep));
    if (U == 8) {
      st.wsc = *reinterpret_cast<const v4i*>(werow + (int64_t)b * (w_packed ? wtiles * 256 : 16));
    } else {  // U == 4: 8 scale bytes
      const v2i t = *reinterpret_cast<const v2i*>(werow + (w_packed ? (int64_t)(b >> 1) * wtiles * 256 + (b & 1) * 8
                                                                     : (int64_t)b * 8));
      st.wsc[0] = t[0];
      st.wsc[1] = t[1];
    }
    const uint8_t* src = qop + (int64_t)b * (U * C::kStepA);  // the batch's operands are contiguous
#pragma unroll
    for (int i = 0; i < C::kStageA; ++i) st.a[i] = *reinterpret_cast<const v4i*>(src + (tid + i * kMidThreads) * 16);
    // scale dwords: 256 of each step's 512-byte record, one 16-byte chunk per thread
    if (tid < U * 16)
      st.asc = *reinterpret_cast<const v4i*>(sa_t + ((int64_t)b * U + (tid >> 4)) * 512 + (tid & 15) * 16);
  };
  auto store_batch = [&](int buf, const Stage& st) __attribute__((always_inline)) {
    uint8_t* sa = s_mid + buf * C::kBufA;
    uint8_t* sw = s_mid + 2 * C::kBufA + buf * C::kBufW;
#pragma unroll
    for (int i = 0; i < C::kStageW; ++i)
      *reinterpret_cast<v4i*>(sw + wdst[i]) = st.w[i];
#pragma unroll
    for (int i = 0; i < C::kStageA; ++i) *reinterpret_cast<v4i*>(sa + (tid + i * kMidThreads) * 16) = st.a[i];
    if (tid < U * 16) *reinterpret_cast<v4i*>(sa + U * C::kStepA + tid * 16) = st.asc;
  };
  v16f acc[RG];
#pragma unroll
  for (int rg = 0; rg < RG; ++rg)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[rg][r] = 0.f;
  auto multiply = [&](int buf, const v4i& sc) __attribute__((always_inline)) {
    const uint8_t* sa_buf = s_mid + buf * C::kBufA;
    const uint8_t* sw_row = s_mid + 2 * C::kBufA + buf * C::kBufW + (wave * 32 + l32) * C::kRowW + kb * 16;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      // the step's row scales: byte rg of the dword is the scale of row 32 rg + l32 (block kb)
      const int sa = *reinterpret_cast<const int*>(sa_buf + U * C::kStepA + u * 256 + kb * 128 + l32 * 4);
      const int sa2 = sa - shift * 0x01010101;  // beta = alpha / 2^shift (the bytes are >= 4)
      // scale byte of block 2u + kb of the batch
      const uint32_t sw = (uint32_t)(u < 2 ? sc[0] : u < 4 ? sc[1] : u < 6 ? sc[2] : sc[3]);
      const int sb = (int)((sw >> (16 * (u & 1) + 8 * kb)) & 0xFFu);
      const v4i w = *reinterpret_cast<const v4i*>(sw_row + u * 32);
      const v8i bw = {w[0], w[1], w[2], w[3], 0, 0, 0, 0};
#pragma unroll
      for (int rg = 0; rg < RG; ++rg) {
        const uint8_t* rec = sa_buf + u * C::kStepA + rg * C::kGroupA;
#pragma unroll
        for (int comp = 0; comp < 2; ++comp) {
          v8i av;
          if constexpr (A4) {
            const uint4 lo = *reinterpret_cast<const uint4*>(rec + (2 * comp + kb) * 512 + l32 * 16);
            av = v8i{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, 0, 0, 0, 0};
          } else {
            const uint4 lo = *reinterpret_cast<const uint4*>(rec + ((3 * comp + kb) * 32 + l32) * 16);
            const uint2 hi = *reinterpret_cast<const uint2*>(rec + (3 * comp + 2) * 512 + lane * 8);
            av = v8i{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, 0, 0};
          }
          const int s = comp ? sa2 : sa;
          if (rg == 0) acc[rg] = mfma_mid<0, CBSZ>(av, bw, acc[rg], s, sb);
          else if (rg == 1) acc[rg] = mfma_mid<1, CBSZ>(av, bw, acc[rg], s, sb);
          else if (rg == 2) acc[rg] = mfma_mid<2, CBSZ>(av, bw, acc[rg], s, sb);
          else acc[rg] = mfma_mid<3, CBSZ>(av, bw, acc[rg], s, sb);
        }
      }
      // four row groups: keep the K steps apart in the schedule, or the hoisted fragment reads spill
      if (RG == 4) __builtin_amdgcn_sched_barrier(0);
    }
  };

  // LDS buffer b % 2 and register stage b % 2 belong to batch b; the scale bytes of a batch stay in
  // a register copy until the batch has been multiplied
  v4i sc_cur = {0, 0, 0, 0}, sc_next = {0, 0, 0, 0};
  load_batch(0, st0);
  if (NB > 1) load_batch(1, st1);
  store_batch(0, st0);
  sc_cur = st0.wsc;
  __syncthreads();
  for (int b = 0; b < NB; b += 2) {
    // even batch in LDS buffer 0; batch b + 1 is in flight into st1
    if (b + 2 < NB) load_batch(b + 2, st0);
    multiply(0, sc_cur);
    if (b + 1 < NB) {
      store_batch(1, st1);
      sc_next = st1.wsc;
    }
    __syncthreads();
    if (b + 1 >= NB) break;
    // odd batch in LDS buffer 1; batch b + 2 is in flight into st0
    if (b + 3 < NB) load_batch(b + 3, st1);
    multiply(1, sc_next);
    if (b + 2 < NB) {
      store_batch(0, st0);
      sc_cur = st0.wsc;
    }
    __syncthreads();
  }
  // D: column l%32, row 8*(r/4) + 4*(l/32) + r%4 in register r
  if (n < N) {
#pragma unroll
    for (int rg = 0; rg < RG; ++rg)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = 32 * rg + 8 * (r >> 2) + 4 * kb + (r & 3);
        if (m < M) {
          if (out_bf16)
            reinterpret_cast<uint16_t*>(y)[(int64_t)m * ldy + n] = f32_to_bf16_bits(acc[rg][r]);
          else
            reinterpret_cast<float*>(y)[(int64_t)m * ldy + n] = acc[rg][r];
        }
      }
  }
}

// ------------------------------------------------------------------ up to 32 rows on packed weights
// The packed layout (msd_pack_weights_w4) holds the B operand of the 32x32x64 instruction as two contiguous
// 512-byte runs per wave and K step (the halves of the kilobytes of two adjacent channel tiles), so the weights go
// HBM -> registers in operand order with no LDS stage: a wave keeps three batches of eight K steps (24 KB) in
// flight in four rotating register sets while it multiplies the fourth.  The activation operands (shared by the
// four waves, hot in L2) still go through LDS, double-buffered, one barrier per batch.
constexpr int kMidpU = 8;          // K steps per batch
constexpr int kMidpSets = 4;       // weight register sets (batches b .. b+3)
constexpr int kMidpStepA = 3072;   // operand bytes of the 32-row group per K step
constexpr int kMidpBufA = kMidpU * (kMidpStepA + 256);
constexpr int kMidpStageA = kMidpU * kMidpStepA / 16 / kMidThreads;  // 16-byte operand chunks per thread and batch
static_assert(kMidpStageA * kMidThreads * 16 == kMidpU * kMidpStepA, "operand staging split");

__global__ __launch_bounds__(kMidThreads) void gemm_w4_midp_kernel(const uint8_t* __restrict__ qop,
                                                                   const uint8_t* __restrict__ sa_t,
                                                                   const uint8_t* __restrict__ Wp,
                                                                   const uint8_t* __restrict__ Ep, void* y,
                                                                   int out_bf16, int64_t ldy, int M, int64_t K,
                                                                   int64_t N, int shift) {
  constexpr int U = kMidpU;
  extern __shared__ __attribute__((aligned(16))) uint8_t s_midp[];  // [2][A batch]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, kb = lane >> 5;
  const int64_t n0 = (int64_t)blockIdx.x * kMidBN;
  const int64_t n = n0 + wave * 32 + l32;
  const int64_t wtiles = (N + 15) / 16, wq = wtiles * 1024;
  const int64_t nc = min(n, N - 1);  // channels past N repeat the last one; their results are not stored
  // this lane's 16 bytes of K step ks: unit ks / 2, half ks % 2 of the kilobyte of its channel tile
  const uint8_t* wl = Wp + (nc / 16) * 1024 + (kb * 16 + (nc & 15)) * 16;
  const uint8_t* el = Ep + (nc / 16) * 256 + (nc & 15) * 16;  // + batch * wtiles * 256: the 16 scale bytes of the batch
  const int NB = (int)(K / (64 * U));
  struct WSet {
    v4i w[U], sc;
  };
  struct ASet {
    v4i a[kMidpStageA], asc;
  };
  WSet w0, w1, w2, w3;
  ASet as;  // one staging set: batch b + 1 is fetched at the start of phase b and written to LDS at its end
  as.asc = v4i{0, 0, 0, 0};
  auto load_w = [&](int b, WSet& ws) __attribute__((always_inline)) {
    const uint8_t* src = wl + (int64_t)b * (U / 2) * wq;
#pragma unroll
    for (int u = 0; u < U; ++u)
      ws.w[u] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(src + (int64_t)(u >> 1) * wq + (u & 1) * 512));
    ws.sc = *reinterpret_cast<const v4i*>(el + (int64_t)b * wtiles * 256);
  };
  auto load_a = [&](int b) __attribute__((always_inline)) {
    const uint8_t* src = qop + (int64_t)b * (U * kMidpStepA);  // the batch's operands are contiguous
#pragma unroll
    for (int i = 0; i < kMidpStageA; ++i) as.a[i] = *reinterpret_cast<const v4i*>(src + (tid + i * kMidThreads) * 16);
    if (tid < U * 16)
      as.asc = *reinterpret_cast<const v4i*>(sa_t + ((int64_t)b * U + (tid >> 4)) * 512 + (tid & 15) * 16);
  };
  auto store_a = [&](int buf) __attribute__((always_inline)) {
    uint8_t* sa = s_midp + buf * kMidpBufA;
#pragma unroll
    for (int i = 0; i < kMidpStageA; ++i) *reinterpret_cast<v4i*>(sa + (tid + i * kMidThreads) * 16) = as.a[i];
    if (tid < U * 16) *reinterpret_cast<v4i*>(sa + U * kMidpStepA + tid * 16) = as.asc;
  };
  v16f acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  // One wave per SIMD: nothing hides an LDS read but the wave's own MFMAs, so the fragments of K step u + 2 are
  // requested before the MFMAs of step u (three rotating fragment sets); left alone the compiler requests all 32
  // reads of a batch up front, and the 96 registers that takes push the weight sets out of the VGPRs.
  struct Frag {
    v8i av[2];
    int sa;
  };
  auto multiply = [&](int buf, const WSet& ws) __attribute__((always_inline)) {
    const uint8_t* sa_buf = s_midp + buf * kMidpBufA;
    auto read_frag = [&](int u, Frag& f) __attribute__((always_inline)) {
      const uint8_t* rec = sa_buf + u * kMidpStepA;
#pragma unroll
      for (int comp = 0; comp < 2; ++comp) {
        const uint4 lo = *reinterpret_cast<const uint4*>(rec + ((3 * comp + kb) * 32 + l32) * 16);
        const uint2 hi = *reinterpret_cast<const uint2*>(rec + (3 * comp + 2) * 512 + lane * 8);
        f.av[comp] = v8i{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, 0, 0};
      }
      // the step's row scales: byte 0 of the dword is the scale of row l32 (block kb)
      f.sa = *reinterpret_cast<const int*>(sa_buf + U * kMidpStepA + u * 256 + kb * 128 + l32 * 4);
    };
    Frag f[3];
    read_frag(0, f[0]);
    read_frag(1, f[1]);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      __builtin_amdgcn_sched_barrier(0);
      if (u + 2 < U) read_frag(u + 2, f[(u + 2) % 3]);
      __builtin_amdgcn_sched_barrier(0);
      const Frag& c = f[u % 3];
      const int sa2 = c.sa - shift * 0x01010101;  // beta = alpha / 2^shift (the bytes are >= 4)
      const uint32_t sw = (uint32_t)(u < 2 ? ws.sc[0] : u < 4 ? ws.sc[1] : u < 6 ? ws.sc[2] : ws.sc[3]);
      const int sb = (int)((sw >> (16 * (u & 1) + 8 * kb)) & 0xFFu);  // scale byte of block 2u + kb of the batch
      const v8i bw = {ws.w[u][0], ws.w[u][1], ws.w[u][2], ws.w[u][3], 0, 0, 0, 0};
      acc = mfma_mid<0, 2>(c.av[0], bw, acc, c.sa, sb);
      acc = mfma_mid<0, 2>(c.av[1], bw, acc, sa2, sb);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  // batch b: weights in register set b % 4, operands in LDS buffer b % 2
  load_a(0);
  load_w(0, w0);
  if (NB > 1) load_w(1, w1);
  if (NB > 2) load_w(2, w2);
  store_a(0);
  __syncthreads();
  // (The load conditions stay in: a steady-state loop peeled into straight-line code made the compiler hoist a
  // whole batch of loads and spill 1.2 KB per lane.)
  auto phase = [&](int b, WSet& cur, WSet& far, int buf) __attribute__((always_inline)) {
    // operands first: loads complete in order, and the operands are needed at the end of this phase, the weights
    // three phases from now
    if (b + 1 < NB) load_a(b + 1);
    if (b + 3 < NB) load_w(b + 3, far);  // the set of batch b - 1, multiplied in the previous phase
    multiply(buf, cur);
    if (b + 1 < NB) store_a(buf ^ 1);    // everyone left that buffer at the last barrier
    __syncthreads();
  };
  for (int b = 0; b < NB; b += 4) {
    phase(b, w0, w3, 0);
    if (b + 1 < NB) phase(b + 1, w1, w0, 1);
    if (b + 2 < NB) phase(b + 2, w2, w1, 0);
    if (b + 3 < NB) phase(b + 3, w3, w2, 1);
  }
  // D: column l%32, row 8*(r/4) + 4*(l/32) + r%4 in register r
  if (n < N) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = 8 * (r >> 2) + 4 * kb + (r & 3);
      if (m < M) {
        if (out_bf16)
          reinterpret_cast<uint16_t*>(y)[(int64_t)m * ldy + n] = f32_to_bf16_bits(acc[r]);
        else
          reinterpret_cast<float*>(y)[(int64_t)m * ldy + n] = acc[r];
      }
    }
  }
}

static int launch_midp(const uint8_t* qop, const uint8_t* sa_t, const uint8_t* Wp, const uint8_t* Ep, void* y,
                       int out_bf16, int64_t ldy, int64_t M, int64_t K, int64_t N, int shift, hipStream_t stream) {
  constexpr int lds = 2 * kMidpBufA;
  hipLaunchKernelGGL(gemm_w4_midp_kernel, dim3((unsigned)cdiv(N, kMidBN)), dim3(kMidThreads), lds, stream, qop, sa_t,
                     Wp, Ep, y, out_bf16, ldy, (int)M, K, N, shift);
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

template <int RG, int U, bool A4>
int launch_mid(const uint8_t* qop, const uint8_t* sa_t, const uint8_t* W, const uint8_t* We, void* y, int out_bf16,
               int64_t ldy, int64_t M, int64_t K, int64_t N, int shift, int w_packed, hipStream_t stream) {
  constexpr int lds = MidCfg<RG, U, A4>::kLds;
  const void* fn = reinterpret_cast<const void*>(&gemm_w4_mid_kernel<RG, U, A4>);
  static bool attr_set = false;
  if (!attr_set) {
    MSD_HIP_CHECK(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    attr_set = true;
  }
  hipLaunchKernelGGL((gemm_w4_mid_kernel<RG, U, A4>), dim3((unsigned)cdiv(N, kMidBN)), dim3(kMidThreads), lds, stream,
                     qop, sa_t, W, We, y, out_bf16, ldy, (int)M, K, N, shift, w_packed);
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

}  // namespace

bool gemm_w4_mid_applies(int64_t M, int64_t K, int64_t N, bool scales_aligned) {
  // whole batches of 8 K steps (4 would do above 32 rows; one rule keeps the layout choice simple);
  // 16-byte loads of the weight scale rows
  return M > 4 && M <= 128 && N >= 1 && K >= 512 && K % 512 == 0 && scales_aligned;
}

W4MidLayout w4_mid_layout(int64_t M, int64_t K) {
  W4MidLayout l{};
  const size_t steps = (size_t)K / 64;
  l.Mpad = M <= 32 ? 32 : M <= 64 ? 64 : 128;
  size_t off = 0;
  l.qop = off; off = align_up(off + steps * (l.Mpad / 32) * 3072, 256);
  l.sa_t = off; off = align_up(off + steps * 512, 256);
  l.total = off;
  return l;
}

int launch_gemm_w4_mid(const uint16_t* x, int64_t ldx, const uint8_t* W, const uint8_t* We, void* y, int out_bf16,
                       int64_t ldy, int64_t M, int64_t K, int64_t N, uint8_t* ws, MxVariant mv, int w_packed,
                       hipStream_t stream) {
  const W4MidLayout l = w4_mid_layout(M, K);
  if (int rc = launch_decompose_mxfp4_pair(x, ldx, M, K, (int64_t)l.Mpad, ws + l.qop, ws + l.sa_t, mv, stream)) return rc;
  const uint8_t* qop = ws + l.qop;
  const uint8_t* sa = ws + l.sa_t;
  if (mv.e2m1) {  // E2M1-grid components as native FP4 operands
    if (l.Mpad == 32) return launch_mid<1, 8, true>(qop, sa, W, We, y, out_bf16, ldy, M, K, N, mv.shift, w_packed, stream);
    if (l.Mpad == 64) return launch_mid<2, 4, true>(qop, sa, W, We, y, out_bf16, ldy, M, K, N, mv.shift, w_packed, stream);
    return launch_mid<4, 4, true>(qop, sa, W, We, y, out_bf16, ldy, M, K, N, mv.shift, w_packed, stream);
  }
  if (l.Mpad == 32 && w_packed) return launch_midp(qop, sa, W, We, y, out_bf16, ldy, M, K, N, mv.shift, stream);
  if (l.Mpad == 32) return launch_mid<1, 8, false>(qop, sa, W, We, y, out_bf16, ldy, M, K, N, mv.shift, w_packed, stream);
  if (l.Mpad == 64) return launch_mid<2, 4, false>(qop, sa, W, We, y, out_bf16, ldy, M, K, N, mv.shift, w_packed, stream);
  return launch_mid<4, 4, false>(qop, sa, W, We, y, out_bf16, ldy, M, K, N, mv.shift, w_packed, stream);
}

}  // namespace msd
