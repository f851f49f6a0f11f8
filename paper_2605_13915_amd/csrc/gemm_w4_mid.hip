// W4A16 MSD GEMM for 3 to 128 activation rows, where the weight stream is the bound (batched
// decode): paper Sec. 3.2.1 / Alg. 2 feeding Sec. 3.4.1 on v_mfma_scale_f32_32x32x64_f8f6f4.
//
// Two launches per call: the K-step-major decomposition of gemm_w4_prefill.hip (per group of 32
// rows 3 KB of FP6 operands per K step of 64 elements, plus one scale record per K step), then one of
// the two kernels of this file: gemm_w4_midp_kernel (further down; weights straight into operand
// registers, hand-counted loads, packed or canonical weight layout) serves the product path;
// gemm_w4_mid_kernel, the first version, described next, remains for the E2M1-grid ablation and for
// weight arrays past 4 GiB.
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
      if (RG >= 3) __builtin_amdgcn_sched_barrier(0);
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

// ------------------------------------------------------------------ 3..128 rows on packed weights
// The packed layout (msd_pack_weights_w4) holds the B operand of the 32x32x64 instruction as two contiguous
// 512-byte runs per wave and K step (the halves of the kilobytes of two adjacent channel tiles), so the weights go
// HBM -> registers in operand order with no LDS stage, in batches of eight K steps (8 KB per wave).  The activation
// operands (shared by the four multiplying waves, hot in L2) go through LDS, filled by four loader waves.  Left
// alone the compiler requests all LDS reads of a batch up front; here the operands of MFMA t + 4 are requested before
// MFMA t (a rotating window of five six-register operands), which also keeps every instance under 256 registers so
// that the loader waves fit beside the multiplying ones.
constexpr int kMidpGroupA = 3072;  // operand bytes of a 32-row group per K step
constexpr int kMidpDepth = 2;      // batches in flight behind the current one (3 measured 2 % slower, 4 spills)
// RG groups of 32 rows, U K steps per batch: 8 steps for one or two groups, 4 for four (three LDS buffers of a
// batch's operands have to fit)
// H16 (up to 16 rows; one row group, eight steps): only the bytes of rows 0..15 of a group's record come to LDS --
// half the operand traffic.  The record in memory is unchanged; the fills gather its eight pieces (the first half
// of each 512-byte chunk, resp. of each block's part of the chunks with dwords 4, 5) into a packed image per pair of
// K steps: [step 2i: 4 x 256 B][step 2i + 1: 4 x 256 B][step 2i: 4 x 128 B][step 2i + 1: 4 x 128 B], piece 2 c + b
// for component c and block b.
template <int RG, int U, bool H16 = false>
struct MidpCfg {
  static_assert(!H16 || (RG == 1 && U == 8), "the 16-row image is written for one group and eight steps");
  static constexpr int kStepG = RG * kMidpGroupA;        // operand bytes per K step in memory
  static constexpr int kStepA = H16 ? kMidpGroupA / 2 : kStepG;  // ... and in LDS
  static constexpr int kBufA = U * (kStepA + 256);       // a batch: operands, then 256 scale bytes per step
  static constexpr int kStageA = U * kStepA / 1024 / (kMidThreads / 64);  // operand kilobytes per wave and batch
  static constexpr int kScaleLanes = U * 256 / 16 / (kMidThreads / 64);   // lanes of a wave that copy scale bytes
  static constexpr int kLds = (kMidpDepth + 1) * kBufA;
  static_assert(kStageA * (kMidThreads / 64) * 1024 == U * kStepA && kScaleLanes <= 32 && kLds <= 160 * 1024, "batch split");
};

// Every vector-memory load is an asm statement and the waits are written by hand, as in the tile kernels: written
// as plain loads with conditions on the batch number, the compiler lost count of the loads in flight at every join
// and waited for all of them before each batch's MFMAs -- the batch requested a moment earlier included, so each
// batch paid a memory latency (37 against 32 us at 32 x 8192 x 28672).
//   D batches ahead of the MFMAs a wave requests the weights of a batch (nine loads into the register set the
//   batch before the current one has left) and then its share of the batch's operands (seven LDS fills: six
//   operand kilobytes, 512 of the 2048 scale bytes with its first 32 lanes) into one of D + 1 LDS buffers.  The
//   issue order is W0 A0 W1 A1 ... from the first instruction on, so when phase b starts the loads younger than
//   the operands of batch b are the D - 1 batches after it: "vmcnt((D - 1) * 16)" means weights and operands of
//   batch b have landed; the barrier after it publishes the fills of all waves and says that every wave has left
//   the buffer that batch b + D goes into (batch b - 1's).  Batch numbers past the end issue the same number of
//   loads, every lane reading the first 16 bytes of the last batch (one cache line per instruction; what they
//   fetch is never used), so the count holds to the end; the kernel drains everything before its epilogue.
__device__ __forceinline__ void midp_fill16(const uint8_t* gbase, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(voff), "s"(gbase), "s"(lds_addr)
               : "memory", "m0");
}
// the same issued by the lanes of `mask` (a subset of lanes 0..31) only, the others switched off inside the statement
template <uint32_t MASK>
__device__ __forceinline__ void midp_fill16_lanes(const uint8_t* gbase, uint32_t voff, uint32_t lds_addr) {
  uint64_t saved;
  asm volatile("s_mov_b64 %0, exec\n\ts_mov_b32 exec_lo, %4\n\ts_mov_b32 exec_hi, 0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\t"
               "global_load_lds_dwordx4 %1, %2\n\ts_mov_b64 exec, %0"
               : "=&s"(saved)
               : "v"(voff), "s"(gbase), "s"(lds_addr), "n"(MASK)
               : "memory", "m0");
}
__device__ __forceinline__ v4i midp_load16(const uint8_t* gbase, uint32_t voff) {
  v4i r;
  asm volatile("global_load_dwordx4 %0, %1, %2 nt" : "=v"(r) : "v"(voff), "s"(gbase) : "memory");
  return r;
}
__device__ __forceinline__ v4i midp_load16_512(const uint8_t* gbase, uint32_t voff) {
  v4i r;
  asm volatile("global_load_dwordx4 %0, %1, %2 offset:512 nt" : "=v"(r) : "v"(voff), "s"(gbase) : "memory");
  return r;
}
__device__ __forceinline__ uint64_t midp_uniform(uint64_t v) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return ((uint64_t)hi << 32) | lo;
}

// CANON: the canonical layout W [N][K/2], We [N][K/32] (Wp / Ep then point at those).  A load straight into the B
// operand would touch 32 weight rows with 32 bytes each; instead the U loads of a batch fetch whole row segments (16
// lanes x 16 B = the batch's 256 bytes of a channel, four channels per instruction; with four steps per batch 8
// lanes x 16 B, eight channels) -- the same number of loads as on packed weights, so the wait counts are the same
// -- and after the batch's wait the wave turns them into operand order through U KB of LDS of its own (chunk c of
// channel r at chunk position c ^ r: stores and operand reads conflict-free; no barrier, the LDS serves a wave in
// order).
template <int D, int RG, int U, int LW, int WN, bool H16 = false, bool CANON = false>
__global__ __launch_bounds__(kMidThreads + LW * 64) void gemm_w4_midp_kernel(const uint8_t* __restrict__ qop,
                                                                   const uint8_t* __restrict__ sa_t,
                                                                   const uint8_t* __restrict__ Wp,
                                                                   const uint8_t* __restrict__ Ep, void* y,
                                                                   int out_bf16, int64_t ldy, int M, int64_t K,
                                                                   int64_t N, int shift, int bn) {
  // bn: channels per workgroup, a multiple of 16, at most kMidBN (the host picks it so that the grid fills the CUs
  // evenly); a wave still multiplies 32 channels, those past bn or N repeat the workgroup's last one
  using C = MidpCfg<RG, U, H16>;
  constexpr int NSETS = D + 1;  // register sets and LDS buffers: the current batch and D in flight
  static_assert(U == 8 || U == 4, "a batch is a whole or half a 16-block scale record");
  extern __shared__ __attribute__((aligned(16))) uint8_t s_midp[];  // [NSETS][A batch]
  // LW = 4: four further waves issue the operand fills (wave 4 + i those of wave i) and do nothing else: the rate at
  // which a CU pulls data grows with the number of waves that issue loads (8192 x 28672: 37.2 -> 30.6 us at 32 rows,
  // 47.8 -> 36.6 at 64, 70.3 -> 50.2 at 128).  A second wave per SIMD needs the kernel under 256 registers.
  static_assert(LW == 0 || LW == kMidThreads / 64, "one loader wave per multiplying wave, or none");
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave_all = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool loader = LW > 0 && wave_all >= kMidThreads / 64;
  const int wave = loader ? wave_all - kMidThreads / 64 : wave_all;
  const int l32 = lane & 31, kb = lane >> 5;
  const int64_t n0 = (int64_t)blockIdx.x * bn;
  const int64_t n_end = min(n0 + bn, N);  // this workgroup's channels are [n0, n_end)
  const int64_t n_raw = n0 + wave * 32 + l32;
  const int64_t n = n_raw < n_end ? n_raw : N;  // N: not stored
  const int64_t wtiles = (N + 15) / 16, wq = wtiles * 1024;
  const int64_t nc = min(n_raw, n_end - 1);  // their loads repeat an address the workgroup reads anyway
  // this lane's 16 bytes of K step ks: unit ks / 2, half ks % 2 of the kilobyte of its channel tile
  const uint32_t w_lane_off = (uint32_t)((nc / 16) * 1024 + (kb * 16 + (nc & 15)) * 16);
  const uint32_t e_lane_off = (uint32_t)((nc / 16) * 256 + (nc & 15) * 16);
  const int NB = (int)(K / (64 * U));
  const uint32_t lds0 = (uint32_t)(uintptr_t)s_midp;
  struct WSet {
    v4i w[U], sc;
  };
  WSet w[NSETS];
  // CANON: load i of a batch covers channels RPL i .. RPL i + RPL - 1 of the wave's 32 (CPR 16-byte chunks each)
  constexpr int CPR = U * 2, RPL = 64 / CPR;
  uint32_t cw_off[CANON ? U : 1];
  uint32_t ce_off = 0;
  uint8_t* stage = s_midp + NSETS * C::kBufA + wave * (U * 1024);  // CANON: this wave's [32 channels][U * 32 B]
  if constexpr (CANON) {
#pragma unroll
    for (int i = 0; i < U; ++i) {
      const int64_t nr = min(n0 + wave * 32 + RPL * i + lane / CPR, n_end - 1);
      cw_off[i] = (uint32_t)(nr * (K / 2) + (lane % CPR) * 16);
    }
    ce_off = (uint32_t)(nc * (K / 32));
  }
  auto load_w = [&](int b, WSet& ws) __attribute__((always_inline)) {
    if constexpr (CANON) {
      const bool live = b < NB;  // past the end: every lane re-reads the first 16 bytes of the array
      b = min(b, NB - 1);
      const uint8_t* src = reinterpret_cast<const uint8_t*>(midp_uniform(reinterpret_cast<uint64_t>(Wp + (int64_t)b * (U * 32))));
#pragma unroll
      for (int i = 0; i < U; ++i) ws.w[i] = midp_load16(src, live ? cw_off[i] : 0u);
      ws.sc = midp_load16(reinterpret_cast<const uint8_t*>(midp_uniform(reinterpret_cast<uint64_t>(Ep + (int64_t)(b * U / 8) * 16))), live ? ce_off : 0u);
      return;
    }
    // past the end: every lane re-reads the first 16 bytes of the last batch (one cache line per instruction)
    const uint32_t w_off = b < NB ? w_lane_off : 0u, e_off = b < NB ? e_lane_off : 0u;
    b = min(b, NB - 1);
    const uint8_t* src = reinterpret_cast<const uint8_t*>(midp_uniform(reinterpret_cast<uint64_t>(Wp + (int64_t)b * (U / 2) * wq)));
    const uint64_t step = midp_uniform((uint64_t)wq);
#pragma unroll
    for (int u = 0; u < U; u += 2) {
      ws.w[u] = midp_load16(src + (u >> 1) * step, w_off);
      ws.w[u + 1] = midp_load16_512(src + (u >> 1) * step, w_off);
    }
    // the scale record covers eight K steps: with four steps per batch two batches share it
    ws.sc = midp_load16(reinterpret_cast<const uint8_t*>(midp_uniform(reinterpret_cast<uint64_t>(Ep + (int64_t)(b * U / 8) * wtiles * 256))), e_off);
  };
  // the batch's operands are contiguous in qop: fill f copies kilobyte f (wave w: f = w, w + 4, ...); the scale
  // bytes are 256 per K step at 512-byte intervals: piece p = w * kScaleLanes + l of the batch (lane l < kScaleLanes of
  // wave w) is piece p % 16 of step p / 16
  const uint32_t a_lane_off = (uint32_t)(lane * 16);
  // H16: lane -> (piece, 16 bytes of it) in the record of a K step; the second 32 lanes of the 128-byte pieces
  // take the next K step
  const uint32_t h16_lo_off = (uint32_t)((3 * (lane >> 5) + ((lane >> 4) & 1)) * 512 + (lane & 15) * 16);
  const uint32_t h16_hi_off = (uint32_t)((lane >> 5) * C::kStepG + (3 * ((lane >> 4) & 1) + 2) * 512 + ((lane >> 3) & 1) * 256 + (lane & 7) * 16);
  const int sp = wave * C::kScaleLanes + (lane & (C::kScaleLanes - 1));
  const uint32_t s_lane_off = (uint32_t)((sp >> 4) * 512 + (sp & 15) * 16);
  auto fill_a = [&](int b) __attribute__((always_inline)) {
    const uint32_t a_off = b < NB ? a_lane_off : 0u, s_off = b < NB ? s_lane_off : 0u;  // past the end: as above
    const int bb = min(b, NB - 1);
    const uint32_t dst = lds0 + (uint32_t)((b % NSETS) * C::kBufA);
    if constexpr (H16) {
      // wave w gathers the pair of K steps 2 w, 2 w + 1: one instruction per step for the 256-byte pieces, one for
      // the 128-byte pieces of both
      const uint8_t* src = reinterpret_cast<const uint8_t*>(midp_uniform(reinterpret_cast<uint64_t>(qop + (int64_t)bb * (U * C::kStepG) + wave * (2 * C::kStepG))));
      const uint32_t lo_off = b < NB ? h16_lo_off : 0u, hi_off = b < NB ? h16_hi_off : 0u;
      midp_fill16(src, lo_off, dst + (uint32_t)(wave * 3072));
      midp_fill16(src + C::kStepG, lo_off, dst + (uint32_t)(wave * 3072 + 1024));
      midp_fill16(src, hi_off, dst + (uint32_t)(wave * 3072 + 2048));
    } else {
      const uint8_t* src = reinterpret_cast<const uint8_t*>(midp_uniform(reinterpret_cast<uint64_t>(qop + (int64_t)bb * (U * C::kStepA) + wave * 1024)));
#pragma unroll
      for (int i = 0; i < C::kStageA; ++i) midp_fill16(src + i * 4096, a_off, dst + (uint32_t)(wave * 1024 + i * 4096));
    }
    midp_fill16_lanes<(uint32_t)((1ull << C::kScaleLanes) - 1)>(
        reinterpret_cast<const uint8_t*>(midp_uniform(reinterpret_cast<uint64_t>(sa_t + (int64_t)bb * U * 512))), s_off,
        dst + (uint32_t)(U * C::kStepA + wave * C::kScaleLanes * 16));
  };
  constexpr int kLoadsA = C::kStageA + 1, kLoadsW = U + 1;
  // loads of a wave per batch: weights and fills, or (with loader waves) the weights only
  constexpr int kYounger = (D - 1) * (LW ? kLoadsW : kLoadsW + kLoadsA);
  static_assert(D >= 1 && kYounger < 64 && (D - 1) * kLoadsA < 64, "vmcnt is a 6-bit field");
  if constexpr (LW > 0) {
    if (loader) {
      // the same barriers as the multiplying waves: batch b's fills have landed (vmcnt) before barrier b, and after
      // it every wave has left the buffer that batch b + D goes into
#pragma unroll
      for (int j = 0; j < D; ++j) fill_a(j);
      for (int b = 0; b < NB; ++b) {
        asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((D - 1) * kLoadsA) : "memory");
        fill_a(b + D);
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      return;
    }
  }
  v16f acc[RG];
#pragma unroll
  for (int rg = 0; rg < RG; ++rg)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[rg][r] = 0.f;
  auto multiply = [&](int buf, int b, const WSet& ws) __attribute__((always_inline)) {
    const uint8_t* sa_buf = s_midp + buf * C::kBufA;
    // the batch's scale dwords: blocks 4 i .. 4 i + 3 of the record in dword i; with four steps per batch the odd
    // batches take the record's second half
    const bool second = U == 4 && (b & 1);
    const uint32_t sd0 = (uint32_t)(second ? ws.sc[2] : ws.sc[0]), sd1 = (uint32_t)(second ? ws.sc[3] : ws.sc[1]);
    // The operands of one MFMA (a row group's component of a K step: six registers) are the unit of the read-ahead:
    // a window of WN units rotates, unit t + WN - 1 is requested before the MFMA of unit t.
    constexpr int UPS = RG * 2, T = U * UPS;  // units per K step and per batch
    v8i win[WN];
    constexpr int SV = (WN - 1 + UPS - 1) / UPS + 1;  // K steps whose row scales are live at once
    int sav[SV];
    v4i bfr[CANON ? SV : 1];  // CANON: the steps' B operands, read with the row scales
    auto read_unit = [&](int t, v8i& d) __attribute__((always_inline)) {
      const int u = t / UPS, rg = (t / 2) % RG, comp = t & 1;
      uint4 lo;
      uint2 hi;
      if constexpr (H16) {  // lanes of rows 16..31 repeat rows 0..15: their products are never stored
        const uint8_t* rec = sa_buf + (u >> 1) * (2 * C::kStepA);
        lo = *reinterpret_cast<const uint4*>(rec + (u & 1) * 1024 + (2 * comp + kb) * 256 + (l32 & 15) * 16);
        hi = *reinterpret_cast<const uint2*>(rec + 2048 + (u & 1) * 512 + (2 * comp + kb) * 128 + (l32 & 15) * 8);
      } else {
        const uint8_t* rec = sa_buf + u * C::kStepA + rg * kMidpGroupA;
        lo = *reinterpret_cast<const uint4*>(rec + ((3 * comp + kb) * 32 + l32) * 16);
        hi = *reinterpret_cast<const uint2*>(rec + (3 * comp + 2) * 512 + lane * 8);
      }
      d = v8i{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, 0, 0};
      // the step's row scales come with its first unit: byte rg of the dword is the scale of row 32 rg + l32 (block kb)
      if (t % UPS == 0) sav[u % SV] = *reinterpret_cast<const int*>(sa_buf + U * C::kStepA + u * 256 + kb * 128 + l32 * 4);
      if constexpr (CANON)
        if (t % UPS == 0)
          bfr[u % SV] = *reinterpret_cast<const v4i*>(stage + l32 * (CPR * 16) + (((2 * u + kb) ^ l32) & (CPR - 1)) * 16);
    };
#pragma unroll
    for (int t = 0; t < WN - 1; ++t) read_unit(t, win[t]);
#pragma unroll
    for (int t = 0; t < T; ++t) {
      __builtin_amdgcn_sched_barrier(0);
      if (t + WN - 1 < T) read_unit(t + WN - 1, win[(t + WN - 1) % WN]);
      __builtin_amdgcn_sched_barrier(0);
      const int u = t / UPS, rg = (t / 2) % RG, comp = t & 1;
      const int sa1 = sav[u % SV];
      const int sx = comp ? sa1 - shift * 0x01010101 : sa1;  // beta = alpha / 2^shift (the bytes are >= 4)
      const uint32_t sw = u < 2 ? sd0 : u < 4 ? sd1 : (uint32_t)(u < 6 ? ws.sc[2] : ws.sc[3]);
      const int sb = (int)((sw >> (16 * (u & 1) + 8 * kb)) & 0xFFu);  // scale byte of block 2u + kb of the batch
      const v4i bq = CANON ? bfr[(CANON ? u % SV : 0)] : ws.w[u];
      const v8i bw = {bq[0], bq[1], bq[2], bq[3], 0, 0, 0, 0};
      const v8i& av = win[t % WN];
      if (rg == 0) acc[rg] = mfma_mid<0, 2>(av, bw, acc[rg], sx, sb);
      else if (rg == 1) acc[rg] = mfma_mid<1, 2>(av, bw, acc[rg], sx, sb);
      else if (rg == 2) acc[rg] = mfma_mid<2, 2>(av, bw, acc[rg], sx, sb);
      else acc[rg] = mfma_mid<3, 2>(av, bw, acc[rg], sx, sb);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  // the registers of `cur` pass through the wait statement, so that nothing that reads them can be placed above it
  auto wait_batch = [&](WSet& cur) __attribute__((always_inline)) {
    if constexpr (U == 8)
      asm volatile("s_waitcnt vmcnt(%9)\n\ts_barrier"
                   : "+v"(cur.w[0]), "+v"(cur.w[1]), "+v"(cur.w[2]), "+v"(cur.w[3]), "+v"(cur.w[4]), "+v"(cur.w[5]),
                     "+v"(cur.w[6]), "+v"(cur.w[7]), "+v"(cur.sc)
                   : "n"(kYounger)
                   : "memory");
    else
      asm volatile("s_waitcnt vmcnt(%5)\n\ts_barrier"
                   : "+v"(cur.w[0]), "+v"(cur.w[1]), "+v"(cur.w[2]), "+v"(cur.w[3]), "+v"(cur.sc)
                   : "n"(kYounger)
                   : "memory");
  };
  auto phase = [&](int b, WSet& cur, WSet& far) __attribute__((always_inline)) {
    wait_batch(cur);
    if constexpr (CANON) {
#pragma unroll
      for (int i = 0; i < U; ++i) {
        const int r = RPL * i + lane / CPR, c = lane % CPR;
        *reinterpret_cast<v4i*>(stage + r * (CPR * 16) + ((c ^ r) & (CPR - 1)) * 16) = cur.w[i];
      }
    }
    load_w(b + D, far);
    if constexpr (LW == 0) fill_a(b + D);
    multiply(b % NSETS, b, cur);
  };
#pragma unroll
  for (int j = 0; j < D; ++j) {
    load_w(j, w[j]);
    if constexpr (LW == 0) fill_a(j);
  }
  for (int b = 0; b < NB; b += NSETS) {
#pragma unroll
    for (int j = 0; j < NSETS; ++j)
      if (j == 0 || b + j < NB) phase(b + j, w[j], w[(j + D) % NSETS]);
  }
  // everything this wave requested has to land before its LDS and registers are given up
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
  for (int j = 0; j < NSETS; ++j) asm volatile("" : "+v"(w[j].sc));
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

template <int RG, int U, int LW, int WN, bool H16 = false, bool CANON = false, int D = kMidpDepth>
static int launch_midp(const uint8_t* qop, const uint8_t* sa_t, const uint8_t* Wp, const uint8_t* Ep, void* y,
                       int out_bf16, int64_t ldy, int64_t M, int64_t K, int64_t N, int shift, hipStream_t stream) {
  constexpr int lds = (D + 1) * MidpCfg<RG, U, H16>::kBufA + (CANON ? (kMidThreads / 64) * U * 1024 : 0);
  static_assert(lds <= 160 * 1024, "LDS");
  static bool attr_set = false;  // per instantiation
  if (!attr_set) {
    MSD_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_w4_midp_kernel<D, RG, U, LW, WN, H16, CANON>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    attr_set = true;
  }
  // Channels per workgroup: 128, or the multiple of 16 (at least 80) that deals the 16-channel tiles evenly to
  // 256 CUs per round -- 28672 channels: 256 workgroups of 112 instead of 224 of 128 (measured 31.8 against 32.5 us).
  const int64_t tiles = cdiv(N, 16);
  const int64_t rounds = cdiv(tiles, 8 * 256);
  const int64_t tpw = cdiv(tiles, 256 * rounds);
  const int bn = tpw >= 5 ? (int)tpw * 16 : kMidBN;
  hipLaunchKernelGGL((gemm_w4_midp_kernel<D, RG, U, LW, WN, H16, CANON>), dim3((unsigned)cdiv(N, bn)), dim3(kMidThreads + LW * 64), lds,
                     stream, qop, sa_t, Wp, Ep, y, out_bf16, ldy, (int)M, K, N, shift, bn);
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
  // from three rows on (8192 x 28672, packed / canonical weights, us: three rows 27.6 / 41.8 here against 31.6 / 40.9
  // in the register-operand kernel, four rows 27.6 / 41.8 against 34.3 / 44.2; two rows 29.6 / 39.5 there)
  return M > 2 && M <= 128 && N >= 1 && K >= 512 && K % 512 == 0 && scales_aligned;
}

W4MidLayout w4_mid_layout(int64_t M, int64_t K) {
  W4MidLayout l{};
  const size_t steps = (size_t)K / 64;
  l.Mpad = M <= 32 ? 32 : M <= 64 ? 64 : M <= 96 ? 96 : 128;
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
    if (l.Mpad == 96) return launch_mid<3, 4, true>(qop, sa, W, We, y, out_bf16, ldy, M, K, N, mv.shift, w_packed, stream);
    return launch_mid<4, 4, true>(qop, sa, W, We, y, out_bf16, ldy, M, K, N, mv.shift, w_packed, stream);
  }
  if (w_packed) {  // weights straight into operand registers, hand-counted loads
    // (one row group: loader waves measured 30.6 against 31.7 us at 32 rows, 28.9 against 30.6 at 8)
    // up to 16 rows: half the operand bytes per K step (8192 x 28672: 28.0 -> 26.1 us at 8 rows, 28.5 -> 26.8 at 16)
    if (M <= 16) return launch_midp<1, 8, 4, 5, true>(qop, sa, W, We, y, out_bf16, ldy, M, K, N, mv.shift, stream);
    if (l.Mpad == 32) return launch_midp<1, 8, 4, 5>(qop, sa, W, We, y, out_bf16, ldy, M, K, N, mv.shift, stream);
    if (l.Mpad == 64) return launch_midp<2, 8, 4, 5>(qop, sa, W, We, y, out_bf16, ldy, M, K, N, mv.shift, stream);
    if (l.Mpad == 96) return launch_midp<3, 4, 4, 5>(qop, sa, W, We, y, out_bf16, ldy, M, K, N, mv.shift, stream);
    return launch_midp<4, 4, 4, 5>(qop, sa, W, We, y, out_bf16, ldy, M, K, N, mv.shift, stream);
  }
  // canonical layout: the same kernel with the weights turned into operand order in LDS; its loads address the
  // array with 32-bit offsets
  if (N * (K / 2) < ((int64_t)1 << 32)) {
    if (M <= 16) return launch_midp<1, 8, 4, 5, true, true>(qop, sa, W, We, y, out_bf16, ldy, M, K, N, mv.shift, stream);
    if (l.Mpad == 32) return launch_midp<1, 8, 4, 5, false, true>(qop, sa, W, We, y, out_bf16, ldy, M, K, N, mv.shift, stream);
    if (l.Mpad == 64) return launch_midp<2, 4, 4, 5, false, true>(qop, sa, W, We, y, out_bf16, ldy, M, K, N, mv.shift, stream);
    if (l.Mpad == 96) return launch_midp<3, 4, 4, 5, false, true>(qop, sa, W, We, y, out_bf16, ldy, M, K, N, mv.shift, stream);
    // four row groups: LDS holds two operand batches instead of three (one batch in flight), no loader waves (with
    // them this instance spills)
    return launch_midp<4, 4, 0, 5, false, true, 1>(qop, sa, W, We, y, out_bf16, ldy, M, K, N, mv.shift, stream);
  }
  if (l.Mpad == 32) return launch_mid<1, 8, false>(qop, sa, W, We, y, out_bf16, ldy, M, K, N, mv.shift, w_packed, stream);
  if (l.Mpad == 64) return launch_mid<2, 4, false>(qop, sa, W, We, y, out_bf16, ldy, M, K, N, mv.shift, w_packed, stream);
  if (l.Mpad == 96) return launch_mid<3, 4, false>(qop, sa, W, We, y, out_bf16, ldy, M, K, N, mv.shift, w_packed, stream);
  return launch_mid<4, 4, false>(qop, sa, W, We, y, out_bf16, ldy, M, K, N, mv.shift, w_packed, stream);
}

}  // namespace msd
