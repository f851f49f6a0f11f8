// W4A16 MSD GEMM, MFMA-bound regime (many activation rows): paper Sec. 3.2.1 / Alg. 2 feeding
// Sec. 3.4.1, on v_mfma_scale_f32_32x32x64_f8f6f4 with an asynchronous global -> LDS pipeline.
//
// Three launches per call:
//   (1) decompose_mxfp4_pair_kernel: Alg. 2 per 32-element block; writes the FP6-E2M3 operands of
//       both components K-step-major and already in the GEMM's LDS order, so that the GEMM copies
//       them with perfectly contiguous 1 KB fetches (the rate of the global -> LDS path falls with
//       the number of cache lines an instruction touches):
//         qop[K step][group of 32 rows][6 chunks of 512 B]
//         chunk 3c+b = [32 rows][dwords 0..3 of block b of component c], chunk 3c+2 = [block][32 rows][dwords 4,5]
//       and the alpha bytes as sa_t[K step][tile of 256 rows][512 B], byte h*256 + b*128 + l*4 + i
//       for row h*128 + 32*i + l of the tile and block b: the four row fragments of a 128-row half share a
//       dword per lane; a wave reads the bytes of its fragments and picks one with the instruction's op_sel.
//   (2) transpose_w_scales_kernel: the weights' E8M0 bytes [N][K/32] -> sw_t in the same layout
//       over columns (the weight values themselves are consumed where they are).
//   (3) gemm_w4_dma_kernel: 256 x 256 output tile, 8 waves of 64 x 128, one K step = 64 elements
//       = two MX blocks = exactly one MFMA K extent (lane l: row/column l%32, block l/32).  A stage
//       is 33 KB: 24 KB activation operands, 8 KB weights, 1 KB scale bytes, filled by 40
//       global_load_lds_dwordx4 instructions (5 per wave: three activation kilobytes, one weight kilobyte,
//       128 bytes of the scales), NS stages deep.  Both components accumulate into the same fp32 accumulator (scale bytes alpha and
//       alpha - 4, i.e. beta = alpha / 16), so the 256 x 256 tile needs 128 accumulator registers per lane.
//
// LDS layout of a stage (every fragment read is linear in the lane, hence conflict-free):
//   activations: 8 groups of 32 rows, each 6 chunks of 512 B as in qop;
//   weights:     8 groups of 32 columns, group = [2 blocks][32 columns][16 B] (= lane order);
//   scales:      512 B for the rows, 512 B for the columns, layout as in sa_t.
#include "decompose_mxfp4_dev.hpp"
#include "kernels.hpp"
#include <type_traits>

namespace msd {

// ------------------------------------------------------------------ (1) decomposition, K-step pairs
__device__ __forceinline__ int scale_slot(int r, int b) {  // byte of (row or column r of a 256 tile, block b)
  return (r >> 7) * 256 + b * 128 + (r & 31) * 4 + ((r >> 5) & 3);
}

__global__ __launch_bounds__(256) void decompose_mxfp4_pair_kernel(const uint16_t* __restrict__ x, int64_t ldx,
                                                                   int64_t M, int KB2, int64_t Mpad,
                                                                   uint32_t* __restrict__ qop,
                                                                   uint8_t* __restrict__ sa_t, int aligned,
                                                                   MxVariant mv) {
  // one thread per (K step, block of the step, row), rows fastest: the 16-byte stores of
  // consecutive threads are adjacent
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= 2 * M * KB2) return;
  const int64_t m = gid % M;
  const int b = (int)((gid / M) & 1);
  const int s = (int)(gid / (2 * M));
  const uint16_t* xb = x + m * ldx + ((int64_t)2 * s + b) * 32;
  uint32_t w[16];
  if (aligned) {
    const uint4* q = reinterpret_cast<const uint4*>(xb);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint4 v = q[i];
      w[4 * i] = v.x; w[4 * i + 1] = v.y; w[4 * i + 2] = v.z; w[4 * i + 3] = v.w;
    }
  } else {
#pragma unroll
    for (int i = 0; i < 16; ++i) w[i] = (uint32_t)xb[2 * i] | ((uint32_t)xb[2 * i + 1] << 16);
  }
  if (mv.e2m1) {
    // native FP4 operands: the 32 E2M1 nibbles of the block, element i at bits [4i, 4i+4) (the ABI order),
    // row m % 32 of chunk 2c + b of the group's four 512-byte chunks
    int k1[32], k2[32];
    const int e4 = mx_block_codes(w, k1, k2, mv);
    uint32_t c1[4], c2[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      uint32_t pa = 0, pc = 0;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        pa |= nibble4(k1[j * 8 + i]) << (4 * i);
        pc |= nibble4(k2[j * 8 + i]) << (4 * i);
      }
      c1[j] = pa;
      c2[j] = pc;
    }
    uint8_t* g4 = reinterpret_cast<uint8_t*>(qop) + (((int64_t)s * (Mpad / 32) + m / 32) * 4) * 512 + (m % 32) * 16;
    *reinterpret_cast<uint4*>(g4 + (0 + b) * 512) = make_uint4(c1[0], c1[1], c1[2], c1[3]);
    *reinterpret_cast<uint4*>(g4 + (2 + b) * 512) = make_uint4(c2[0], c2[1], c2[2], c2[3]);
    uint8_t* sc4 = sa_t + ((int64_t)s * max(Mpad / 256, (int64_t)1) + m / 256) * 512;
    sc4[scale_slot((int)(m % 256), b)] = (uint8_t)(e4 + 127);
    return;
  }
  uint32_t p1[6], p2[6];
  const int e = mx_block_pack_fp6(w, p1, p2, mv);
  // group of 32 rows: 6 chunks of 512 B; this block's dwords 0..3 fill row m % 32 of chunk 3c + b
  // ([32 rows][16 B]), its dwords 4, 5 row m % 32 of half b of chunk 3c + 2 ([2 blocks][32 rows][8 B])
  uint8_t* g = reinterpret_cast<uint8_t*>(qop) + (((int64_t)s * (Mpad / 32) + m / 32) * 6) * 512;
  const int r = (int)(m % 32);
  *reinterpret_cast<uint4*>(g + (0 + b) * 512 + r * 16) = make_uint4(p1[0], p1[1], p1[2], p1[3]);
  *reinterpret_cast<uint2*>(g + 2 * 512 + b * 256 + r * 8) = make_uint2(p1[4], p1[5]);
  *reinterpret_cast<uint4*>(g + (3 + b) * 512 + r * 16) = make_uint4(p2[0], p2[1], p2[2], p2[3]);
  *reinterpret_cast<uint2*>(g + 5 * 512 + b * 256 + r * 8) = make_uint2(p2[4], p2[5]);
  uint8_t* sc = sa_t + ((int64_t)s * max(Mpad / 256, (int64_t)1) + m / 256) * 512;
  sc[scale_slot((int)(m % 256), b)] = (uint8_t)(e + 127);
}

// ------------------------------------------------------------------ (2) weight scale bytes, K-step-major
// One workgroup moves a 64 (columns) x 64 (K steps) tile of byte pairs through LDS so that both the
// reads (along K) and the writes (along N) are contiguous.
__global__ __launch_bounds__(256) void transpose_w_scales_kernel(const uint8_t* __restrict__ We, int64_t N,
                                                                 int KB2, int64_t Npad,
                                                                 uint8_t* __restrict__ sw_t) {
  __shared__ uint16_t tile[64][65];
  const int64_t n0 = (int64_t)blockIdx.x * 64;
  const int s0 = blockIdx.y * 64;
  for (int i = threadIdx.x; i < 64 * 64; i += 256) {
    const int r = i >> 6, c = i & 63;  // r: column of W within the tile, c: K step
    const int64_t n = n0 + r;
    const int s = s0 + c;
    uint16_t v = 0x7F7F;
    if (n < N && s < KB2) {
      const uint8_t* p = We + (n * KB2 + s) * 2;
      v = (uint16_t)p[0] | ((uint16_t)p[1] << 8);
    }
    tile[r][c] = v;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 64 * 64; i += 256) {
    const int c = i >> 6, r = i & 63;  // consecutive threads -> consecutive columns of W
    const int64_t n = n0 + r;
    const int s = s0 + c;
    if (n < Npad && s < KB2) {
      uint8_t* sc = sw_t + ((int64_t)s * (Npad / 256) + n / 256) * 512;
      const uint16_t v = tile[r][c];
      sc[scale_slot((int)(n % 256), 0)] = (uint8_t)(v & 0xFF);
      sc[scale_slot((int)(n % 256), 1)] = (uint8_t)(v >> 8);
    }
  }
}

// ------------------------------------------------------------------ (3) GEMM
template <int SELA, int SELB, int CBSZ = 2>
__device__ __forceinline__ v16f mfma64_scaled(v8i a, v8i b, v16f c, int sa, int sb) {
  // A: FP6 E2M3 (cbsz = 2) or FP4 E2M1 (cbsz = 4), B: FP4 E2M1 (blgp = 4); E8M0 scales: byte SELA of sa,
  // byte SELB of sb
  return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, CBSZ, 4, SELA, sa, SELB, sb);
}

__device__ __forceinline__ void w4_lds_dma16(const uint8_t* gbase, uint32_t voff, uint32_t lds_addr) {
  // the base is wave-uniform by construction; say so, or the "s" operand may be given a VGPR pair
  const uint64_t g = reinterpret_cast<uint64_t>(gbase);
  const uint32_t glo = __builtin_amdgcn_readfirstlane((uint32_t)g), ghi = __builtin_amdgcn_readfirstlane((uint32_t)(g >> 32));
  gbase = reinterpret_cast<const uint8_t*>(((uint64_t)ghi << 32) | glo);
  lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(voff), "s"(gbase), "s"(lds_addr)
               : "memory", "m0");
}

// The same instruction issued by lanes 0..7 only (128 bytes): the other lanes are switched off inside the
// statement, so the caller's code stays free of branches.
__device__ __forceinline__ void w4_lds_dma16_lanes8(const uint8_t* gbase, uint32_t voff, uint32_t lds_addr) {
  const uint64_t g = reinterpret_cast<uint64_t>(gbase);
  const uint32_t glo = __builtin_amdgcn_readfirstlane((uint32_t)g), ghi = __builtin_amdgcn_readfirstlane((uint32_t)(g >> 32));
  gbase = reinterpret_cast<const uint8_t*>(((uint64_t)ghi << 32) | glo);
  lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);
  uint64_t saved;
  asm volatile("s_mov_b64 %0, exec\n\ts_mov_b64 exec, 0xff\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\t"
               "global_load_lds_dwordx4 %1, %2\n\ts_mov_b64 exec, %0"
               : "=&s"(saved)
               : "v"(voff), "s"(gbase), "s"(lds_addr)
               : "memory", "m0");
}

template <int N>
__device__ __forceinline__ void w4_wait_vm_barrier() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

constexpr int kW4PGroupM = 8;

// PROBE = true is a measurement aid (msd_probe_mfma_w4a16): after the first K step the kernel stops
// fetching and keeps multiplying that step's operands -- the same scaled-MFMA sequence, tile
// schedule and epilogue on real operand bits, without fill, barriers and LDS traffic.
// A4 = true: the activation components are OCP E2M1 codes (the E2M1-grid ablation) and travel as native
// FP4 operands, 16 bytes per lane and block instead of 24: a group of 32 rows is 2 KB per K step
// (chunk 2c+b = [32 rows][16 B of block b of component c]), a stage 25 KB, 3 fill instructions per wave.
template <int NS, bool PROBE = false, bool A4 = false>
__global__ __launch_bounds__(512) void gemm_w4_dma_kernel(GemmW4PrefillArgs a, int tiles_m, int tiles_n) {
  constexpr int GA = A4 ? 2048 : 3072;  // operand bytes of a 32-row group per K step
  constexpr int CA = GA / 2;            // of one component
  constexpr int SZ_A = 8 * GA, SZ_W = 8192, STAGE = SZ_A + SZ_W + 1024;
  constexpr int QA = SZ_A / 8192;       // activation fill instructions per wave and stage
  constexpr int L = QA + 2;             // load instructions per wave and stage: QA activation, 1 weight, 1 scale piece
  constexpr int CBSZ = A4 ? 4 : 2;
  static_assert(NS >= 3 && (NS - 2) * L < 64, "stage count");
  extern __shared__ __attribute__((aligned(16))) uint8_t smem4p[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // eight waves, 64 rows x 128 columns each: of the shapes with 128 accumulator registers the one that reads the
  // fewest operand bytes from LDS per K step (10 KB per wave; 128 x 64 reads 14 KB -- the 6-bit activation
  // operands of two components are three times the bytes of the 4-bit weights)
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, kb = lane >> 5;
  const int64_t M = a.M, N = a.N;
  const int KT = (int)(a.K / 64);
  const uint32_t step_a = (uint32_t)(a.Mpad * (GA / 32));  // bytes of qop per K step
  const int64_t row_w = a.K / 2;           // bytes per weight row
  const int total = tiles_m * tiles_n;
  int id = blockIdx.x;
  {
    const int per_xcd = (total + 7) / 8;
    id = (id % 8) * per_xcd + id / 8;
  }
  if (id >= total) return;
  const int group = id / (kW4PGroupM * tiles_n);
  const int first_m = group * kW4PGroupM;
  const int rows_in_group = min(kW4PGroupM, tiles_m - first_m);
  const int in_group = id - group * kW4PGroupM * tiles_n;
  const int tm = first_m + in_group % rows_in_group;
  const int tn = in_group / rows_in_group;
  const int64_t m0 = (int64_t)tm * 256, n0 = (int64_t)tn * 256;

  // ---- this wave's load instructions per stage: instruction idx = q*8 + wave of the 32 data
  // instructions.  The stage image is linear in idx (24 KB of activation operands, then 8 weight
  // groups of 1 KB), and so is the activation source (qop holds the tile's 24 KB of a K step
  // contiguously): instruction idx < 24 (q < QA) copies kilobyte idx of it.  Instructions 24..31
  // (q = QA) gather weight group idx - 24 = wave (32 columns x 2 blocks).  All bases are wave-uniform
  // scalars; only the weight offset and the scale offset are per lane.
  const uint32_t lds0 = (uint32_t)(uintptr_t)smem4p;
  const uint8_t* a_src = a.qop + (m0 / 32 * (GA / 1024) + wave) * 1024;  // + kt * step_a + q * 8192, lane * 16
  // packed weights (msd_pack_weights_w4): the 32 columns x 2 blocks of a wave and K step are two 512-byte halves
  // of the kilobytes of two adjacent channel tiles
  const int64_t wtiles = (N + 15) / 16, wq = wtiles * 1024;
  const uint8_t* w_src = a.w_packed ? a.W + (n0 / 16) * 1024 : a.W + n0 * row_w;  // + K step, lane offsets below
  const uint32_t voff_w =
      a.w_packed ? (uint32_t)((min(n0 / 16 + 2 * wave + (l32 >> 4), wtiles - 1) - n0 / 16) * 1024 + (kb * 16 + (l32 & 15)) * 16)
                 : (uint32_t)((min(n0 + 32 * wave + l32, N - 1) - n0) * row_w + kb * 16);
  // bytes from one pair of K steps to the next, and from the even to the odd step of a pair (no branch on the layout
  // inside the K loop)
  const int64_t w_pair = a.w_packed ? wq : 64;
  const int w_odd = a.w_packed ? 512 : 32;
  const uint32_t voff_a = (uint32_t)(lane * 16);
  // scale bytes of a stage: one kilobyte, the 512 bytes of sa_t[kt][tm] then those of sw_t[kt][tn], in 64 pieces
  // of 16 bytes; wave w fetches pieces 8w .. 8w+7 with its lanes 0..7 (waves 0..3 activation scales, 4..7 weight
  // scales), so that every wave issues the same number of loads per stage and waits on the same count
  const int sp = wave * 8 + (lane & 7), skb = sp >> 5, sl = sp & 31;
  const uint8_t* sbase = skb ? a.sw_t : a.sa_t;  // wave-uniform
  const uint64_t s_first = (uint64_t)(skb ? n0 : m0) * 2 + 16 * sl;  // byte offset from sbase (below 2^32: host check)
  const uint64_t s_inc = (uint64_t)(skb ? a.Npad : a.Mpad) * 2;      // per K step
  auto issue_one = [&](int kt, int q) {  // q is a compile-time constant at every call site
    const uint32_t dst = lds0 + (uint32_t)((kt % NS) * STAGE) + (uint32_t)(wave * 1024 + q * 8192);
    if (q < QA) w4_lds_dma16(a_src + (int64_t)kt * step_a + q * 8192, voff_a, dst);
    else if (q == QA)
      w4_lds_dma16(w_src + (int64_t)(kt >> 1) * w_pair + (kt & 1) * w_odd, voff_w, dst);
    else
      w4_lds_dma16_lanes8(sbase, (uint32_t)(s_first + (uint64_t)kt * s_inc),
                          lds0 + (uint32_t)((kt % NS) * STAGE) + SZ_A + SZ_W + (uint32_t)(wave * 128));
  };
  auto issue = [&](int kt) {
#pragma unroll
    for (int q = 0; q < L; ++q) issue_one(kt, q);
  };

  constexpr int FI = 2, FJ = 4;  // row / column fragments of a wave
  v16f acc[FI][FJ];
#pragma unroll
  for (int i = 0; i < FI; ++i)
#pragma unroll
    for (int j = 0; j < FJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // per-lane LDS offsets inside a stage (kb*32 + l32 == lane, so the 16-byte reads are linear in the lane)
  const uint32_t o_main = lane * 16, o_tail = lane * 8, o_sc = kb * 128 + l32 * 4;
  auto load_a = [&](int kt, int c, v8i (&fa)[FI]) {  // component c of K step kt
    const uint8_t* st = smem4p + (kt % NS) * STAGE + wm * (FI * GA) + c * CA;
#pragma unroll
    for (int i = 0; i < FI; ++i) {
      const uint4 v = *reinterpret_cast<const uint4*>(st + i * GA + o_main);
      if constexpr (A4) {
        fa[i] = v8i{(int)v.x, (int)v.y, (int)v.z, (int)v.w, 0, 0, 0, 0};
      } else {
        const uint2 t = *reinterpret_cast<const uint2*>(st + i * GA + 1024 + o_tail);
        fa[i] = v8i{(int)v.x, (int)v.y, (int)v.z, (int)v.w, (int)t.x, (int)t.y, 0, 0};
      }
    }
  };
  // weights and scale bytes of K step kt; sa / sb: byte i = scale of row fragment i / column fragment i
  // (a scale dword holds the four fragments of a 128-row or 128-column half: the wave's two row fragments are
  // one 16-bit read, its four column fragments the whole dword)
  auto load_b = [&](int kt, v8i (&fb)[FJ], int& sa, int& sb) {
    const uint8_t* st = smem4p + (kt % NS) * STAGE;
    // the scale bytes first and without arithmetic on them (this wave's two column bytes are one 16-bit read):
    // whatever waits for them then waits for nothing issued after them
    sa = (int)*reinterpret_cast<const uint16_t*>(st + SZ_A + SZ_W + (wm >> 1) * 256 + (wm & 1) * 2 + o_sc);
    sb = *reinterpret_cast<const int*>(st + SZ_A + SZ_W + 512 + wn * 256 + o_sc);
#pragma unroll
    for (int j = 0; j < FJ; ++j) {
      const uint4 v = *reinterpret_cast<const uint4*>(st + SZ_A + (wn * FJ + j) * 1024 + o_main);
      fb[j] = v8i{(int)v.x, (int)v.y, (int)v.z, (int)v.w, 0, 0, 0, 0};
    }
  };
  // one component block: 8 MFMAs on 8 different accumulators; the first one is issued ahead of
  // the LDS reads that run under the block, so that the compiler's wait for this block's
  // operands (it cannot count LDS operations across the inline asm) covers no read just issued
  auto mfma_first = [&](const v8i (&fa)[FI], const v8i (&fb)[FJ], int sa, int sb) {
    acc[0][0] = mfma64_scaled<0, 0, CBSZ>(fa[0], fb[0], acc[0][0], sa, sb);
  };
  // ISSUE: the load instructions of tile kt_issue go out between the MFMAs, one after every second
  // MFMA (in one burst after the barrier they fill the address queue, the waves leave the burst at
  // different times and the next barrier pays for the skew); the scale piece goes last.
  // do_issue: a bool, or std::true_type where the loads are unconditional (the steady state of the K loop, which
  // must stay one basic block: across a branch the compiler sinks the MFMAs below the fragment reads, the barrier
  // and the loads, and nothing overlaps any more).  Loads 0..3 follow MFMAs 1, 3, 5, 7, load 4 follows MFMA 6.
  auto mfma_rest = [&](const v8i (&fa)[FI], const v8i (&fb)[FJ], int sa, int sb, int kt_issue, auto do_issue) {
    auto post = [&](auto idx) {
      constexpr int IDX = decltype(idx)::value;
      constexpr int q = (IDX % 2 == 0) ? IDX / 2 : (IDX == 5 ? 4 : -1);
      if constexpr (q >= 0 && q < L) {
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (std::is_same_v<decltype(do_issue), std::true_type>) {
          issue_one(kt_issue, q);
        } else {
          if (do_issue) issue_one(kt_issue, q);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    // MFMA number I * FJ + J multiplies row fragment I by column fragment J; number 0 is mfma_first
#define MSD_W4_MM(I, J)                                                                  \
  acc[I][J] = mfma64_scaled<I, J, CBSZ>(fa[I], fb[J], acc[I][J], sa, sb);                \
  post(std::integral_constant<int, (I) * FJ + (J) - 1>{});
    MSD_W4_MM(0, 1) MSD_W4_MM(0, 2) MSD_W4_MM(0, 3) MSD_W4_MM(1, 0) MSD_W4_MM(1, 1) MSD_W4_MM(1, 2) MSD_W4_MM(1, 3)
#undef MSD_W4_MM
    static_assert(L <= 5, "load slots between the eight MFMAs of a block");
  };
  // wait until tile t has landed (the tiles issued after it may stay in flight), then barrier
  auto wait_tile = [&](int t, int newest_issued) {
    const int younger = newest_issued - t;
    if (younger == NS - 2) w4_wait_vm_barrier<(NS - 2) * L>();
    else if (younger == NS - 3) w4_wait_vm_barrier<(NS - 3) * L>();
    else w4_wait_vm_barrier<0>();
  };

  // Pipeline of K step s:  block 0 = component 1 ... the registers roll as follows.
  //   first block  (component 0 of step s): under it the component-1 operands of step s are read;
  //   barrier for tile s+1; the stage of tile s-1 is free now and is refilled with tile s-1+NS;
  //   second block (component 1 of step s): under it the component-0 operands, the weights and
  //   the scale bytes of step s+1 are read (weights and scales are double-buffered in registers,
  //   the activation operands are not: each set is dead when its successor is fetched).
  v8i a0[FI], a1[FI], b0[FJ], b1[FJ];
  int sa0 = 0, sb0 = 0, sa1 = 0, sb1 = 0;
  const int beta_shift = a.mv.shift * 0x01010101;
  auto step = [&](auto steady, int s, v8i (&bc)[FJ], int sac, int sbc, v8i (&bn)[FJ], int& san, int& sbn) {
    constexpr bool STEADY = decltype(steady)::value;  // s + NS - 1 < KT: every condition below holds
    if constexpr (PROBE) {
      if (s > 0) {  // operands of step 0 (a1: component 1 of step 0), no data movement
        mfma_first(a0, b0, sa0, sb0);
        mfma_rest(a0, b0, sa0, sb0, 0, false);
        __builtin_amdgcn_sched_barrier(0);
        mfma_first(a1, b0, sa0 - beta_shift, sb0);
        mfma_rest(a1, b0, sa0 - beta_shift, sb0, 0, false);
        __builtin_amdgcn_sched_barrier(0);
        return;
      }
    }
    mfma_first(a0, bc, sac, sbc);
    __builtin_amdgcn_sched_barrier(0);
    load_a(s, 1, a1);
    __builtin_amdgcn_sched_barrier(0);
    mfma_rest(a0, bc, sac, sbc, 0, false);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (STEADY) {
      w4_wait_vm_barrier<(NS - 3) * L>();
    } else {
      if (s + 1 < KT) wait_tile(s + 1, min(KT - 1, s + NS - 2));
    }
    const int sac2 = sac - beta_shift;  // beta = alpha / 2^shift: every scale byte minus shift (bytes are >= 4)
    mfma_first(a1, bc, sac2, sbc);
    __builtin_amdgcn_sched_barrier(0);
    if (STEADY || (!PROBE && s + 1 < KT)) {
      load_b(s + 1, bn, san, sbn);
      load_a(s + 1, 0, a0);
    }
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (STEADY) mfma_rest(a1, bc, sac2, sbc, s - 1 + NS, std::true_type{});
    else mfma_rest(a1, bc, sac2, sbc, s - 1 + NS, !PROBE && s + 1 < KT && s - 1 + NS < KT);
    __builtin_amdgcn_sched_barrier(0);
  };
#pragma unroll
  for (int t = 0; t < NS - 1; ++t)
    if (t < KT) issue(t);
  if (KT > 0) {
    wait_tile(0, min(KT - 1, NS - 2));
    load_a(0, 0, a0);
    load_b(0, b0, sa0, sb0);
  }
  int s = 0;
  if constexpr (!PROBE) {
    for (; s + NS < KT; s += 2) {  // both steps of the pair are in the steady state
      step(std::true_type{}, s, b0, sa0, sb0, b1, sa1, sb1);
      step(std::true_type{}, s + 1, b1, sa1, sb1, b0, sa0, sb0);
    }
  }
  for (; s < KT; s += 2) {
    step(std::false_type{}, s, b0, sa0, sb0, b1, sa1, sb1);
    if (s + 1 < KT) step(std::false_type{}, s + 1, b1, sa1, sb1, b0, sa0, sb0);
  }

  // ---- epilogue: the accumulators are the output (both components and all scales are in them)
#pragma unroll
  for (int i = 0; i < FI; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int64_t m = m0 + wm * 64 + 32 * i + (r >> 2) * 8 + kb * 4 + (r & 3);
      if (m < M) {
#pragma unroll
        for (int j = 0; j < FJ; ++j) {
          const int64_t n = n0 + wn * 128 + 32 * j + l32;
          if (n >= N) continue;
          const float v = acc[i][j][r];
          if (a.out_bf16)  // written once, not read again: streaming stores
            __builtin_nontemporal_store(f32_to_bf16_bits(v), reinterpret_cast<uint16_t*>(a.y) + m * a.ldy + n);
          else
            __builtin_nontemporal_store(v, reinterpret_cast<float*>(a.y) + m * a.ldy + n);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
}

// ------------------------------------------------------------------ host side
bool gemm_w4_prefill_applies(int64_t M, int64_t K, int64_t N) {
  (void)N;
  return M > 32 && K >= 64 && K % 64 == 0;
}

W4PrefillLayout w4_prefill_layout(int64_t M, int64_t K, int64_t N) {
  W4PrefillLayout l{};
  const size_t KB2 = (size_t)K / 64;
  l.Mpad = align_up((size_t)M, 256);
  l.Npad = align_up((size_t)N, 256);
  size_t off = 0;
  l.qop = off; off = align_up(off + l.Mpad * KB2 * 96, 256);
  l.sa_t = off; off = align_up(off + KB2 * l.Mpad * 2, 256);
  l.sw_t = off; off = align_up(off + KB2 * l.Npad * 2, 256);
  l.total = off;
  return l;
}

size_t w4_packed_scales_decode_bytes(int64_t N, int64_t K) {
  return align_up((size_t)((K + 511) / 512) * (size_t)((N + 15) / 16) * 256, 256);
}

size_t w4_packed_scales_bytes(int64_t N, int64_t K) {
  return w4_packed_scales_decode_bytes(N, K) + (size_t)(K / 64) * align_up((size_t)N, 256) * 2;
}

// canonical E8M0 bytes [N][K/32] -> the stage order of the many-row kernel (sw_t above)
int launch_transpose_w_scales(const uint8_t* We, int64_t N, int64_t K, uint8_t* sw_t, hipStream_t stream) {
  const int KB2 = (int)(K / 64);
  const int64_t Npad = (int64_t)align_up((size_t)N, 256);
  hipLaunchKernelGGL(transpose_w_scales_kernel, dim3((unsigned)(Npad / 64), (unsigned)cdiv(KB2, 64)), dim3(256), 0,
                     stream, We, N, KB2, Npad, sw_t);
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

int launch_decompose_mxfp4_pair(const uint16_t* x, int64_t ldx, int64_t M, int64_t K, int64_t Mpad, uint8_t* qop,
                                uint8_t* sa_t, MxVariant mv, hipStream_t stream) {
  const int KB2 = (int)(K / 64);
  const int aligned = ((reinterpret_cast<uintptr_t>(x) & 15) == 0 && (ldx % 8) == 0) ? 1 : 0;
  hipLaunchKernelGGL(decompose_mxfp4_pair_kernel, dim3((unsigned)cdiv(2 * M * KB2, 256)), dim3(256), 0, stream, x, ldx,
                     M, KB2, Mpad, reinterpret_cast<uint32_t*>(qop), sa_t, aligned, mv);
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

int launch_gemm_w4_prefill(const uint16_t* x, int64_t ldx, const uint8_t* W, const uint8_t* We, void* y,
                           int out_bf16, int64_t ldy, int64_t M, int64_t K, int64_t N, uint8_t* ws,
                           MxVariant mv, hipStream_t stream, bool probe, int w_packed) {
  const W4PrefillLayout l = w4_prefill_layout(M, K, N);
  if (l.total >= ((size_t)1 << 31)) return MSD_ERR_UNSUPPORTED;  // 32-bit offsets inside the workspace ...
  if (int rc = launch_decompose_mxfp4_pair(x, ldx, M, K, (int64_t)l.Mpad, ws + l.qop, ws + l.sa_t, mv, stream)) return rc;
  // packed weights carry their scale bytes in this kernel's order already (second part of the packed array)
  if ((size_t)(K / 64) * l.Npad * 2 >= ((size_t)1 << 31)) return MSD_ERR_UNSUPPORTED;  // ... and the scale arrays
  const uint8_t* sw_t = w_packed ? We + w4_packed_scales_decode_bytes(N, K) : ws + l.sw_t;
  if (!w_packed)
    if (int rc = launch_transpose_w_scales(We, N, K, ws + l.sw_t, stream)) return rc;
  GemmW4PrefillArgs a{};
  a.qop = ws + l.qop;
  a.sa_t = ws + l.sa_t;
  a.sw_t = sw_t;
  a.W = W;
  a.w_packed = w_packed;
  a.y = y;
  a.out_bf16 = out_bf16;
  a.ldy = ldy;
  a.M = M; a.K = K; a.N = N;
  a.Mpad = (int64_t)l.Mpad;
  a.Npad = (int64_t)l.Npad;
  a.mv = mv;
  constexpr int NS = 4;
  const int tiles_m = (int)cdiv(M, 256), tiles_n = (int)cdiv(N, 256);
  const int total = tiles_m * tiles_n;
  const int grid = ((total + 7) / 8) * 8;
  const size_t lds = (size_t)NS * (24576 + 8192 + 1024);
  static bool attr_set = false;
  if (!attr_set) {
    MSD_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_w4_dma_kernel<NS, false>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    MSD_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_w4_dma_kernel<NS, true>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    MSD_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_w4_dma_kernel<NS, false, true>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_set = true;
  }
  if (mv.e2m1)  // E2M1-grid components as native FP4 operands (the probe keeps the FP6 form)
    hipLaunchKernelGGL((gemm_w4_dma_kernel<NS, false, true>), dim3(grid), dim3(512),
                       (size_t)NS * (16384 + 8192 + 1024), stream, a, tiles_m, tiles_n);
  else if (probe)
    hipLaunchKernelGGL((gemm_w4_dma_kernel<NS, true>), dim3(grid), dim3(512), lds, stream, a, tiles_m, tiles_n);
  else
    hipLaunchKernelGGL((gemm_w4_dma_kernel<NS, false>), dim3(grid), dim3(512), lds, stream, a, tiles_m, tiles_n);
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

}  // namespace msd
