// W4A16 MSD GEMM for gfx950 (paper Sec. 3.2.1 / Alg. 2 feeding Sec. 3.4.1): both 4-bit
// activation components are multiplied against the MXFP4 weights by the block-scaled MFMA
// v_mfma_scale_f32_16x16x128_f8f6f4 and summed in one fp32 accumulator, so the weights are
// never expanded.
//
// Operand formats.  The paper's activation grid {k/4, |k| <= 7} is uniform, which OCP E2M1
// cannot represent (5/4 and 7/4 are missing), so the activation components travel as
// FP6-E2M3 (an exact superset; magnitude field 2|k|) in the A operand; the weights stay OCP
// E2M1 in the B operand.  Both operands are below 8 bits, so the instruction issues at the
// FP4/FP6 rate.  Block scales are the hardware's E8M0 bytes: alpha (or beta = alpha/16, byte
// minus 4) per activation block, the stored weight scale per weight block.
//
// MFMA layout: lane l holds row/column l%16 and one 32-element K block; the scale byte of a
// lane applies to that block.  Which block a lane group takes is free as long as A and B
// agree: over a super-step of 16 blocks, MFMA u (u = 0..3) gives lane group g = l/16 block
// 4u+g, so the four lanes of a row read 64 contiguous weight bytes per load instruction
// (measured: the transposed assignment 4g+u, 16 bytes out of every 64 per instruction, streamed
// 30 % slower).  The 16 scale bytes of a row and super-step come as one 16-byte load; a lane
// shifts its byte (4u+g) down to bits 7:0.

#include "decompose_mxfp4_dev.hpp"
#include "kernels.hpp"

namespace msd {

__device__ __forceinline__ v4f mfma_scaled(v8i a, v8i b, v4f c, int sa, int sb) {
  // A: FP6 E2M3 (cbsz = 2), B: FP4 E2M1 (blgp = 4); E8M0 scales in byte 0 of sa / sb
  return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 2, 4, 0, sa, 0, sb);
}

// byte 4*d+b of the 16 scale bytes sc[0..3] of a super-step, in bits 7:0
__device__ __forceinline__ int scale_byte(const v4i& sc, int d, int b) {
  const uint32_t w = d == 0 ? sc[0] : d == 1 ? sc[1] : d == 2 ? sc[2] : sc[3];
  return (int)((w >> (8 * b)) & 0xFFu);
}

__device__ __forceinline__ v8i load_fp6_slot(const uint32_t* p) {  // 24 B of a 32 B slot (global)
  const uint4 lo = *reinterpret_cast<const uint4*>(p);
  const uint2 hi = *reinterpret_cast<const uint2*>(p + 4);
  return v8i{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, 0, 0};
}
__device__ __forceinline__ v8i load_fp6_lds(const uint8_t* p) {  // 24 B, 8-byte aligned (LDS)
  const uint2* q = reinterpret_cast<const uint2*>(p);
  const uint2 x0 = q[0], x1 = q[1], x2 = q[2];
  return v8i{(int)x0.x, (int)x0.y, (int)x1.x, (int)x1.y, (int)x2.x, (int)x2.y, 0, 0};
}

// One workgroup: rows [m0, m0 + 16*RT) x 16 output channels; WAVES waves split K in super-steps
// of 16 blocks.  Per batch of U super-steps a wave first issues all its weight loads (HBM ->
// registers in B-operand layout), then fetches the activation operands, then runs the MFMAs.
//
// SELF (M = 1, RT = 1; the kernel itself handles up to two rows): the kernel decomposes the activations itself (Alg. 2) -- the block
// decomposition needs no reduction beyond the 32-element block, so each wave handles exactly the
// blocks of its own K range, one block per lane, into wave-private LDS, under its own weight
// loads.  One launch per call, nothing materialised in HBM.
// FAST: K is a whole number of super-steps and the scale arrays are 16-byte aligned, so no load in
// the main loop is predicated per lane (predicated loads do not batch: measured 25 % slower).
// Rows past M are clamped to the last row (their results are never stored).
// STACK (2M <= 16, RT = 1): the two components share one MFMA -- fragment rows [0, M) carry x1,
// rows [M, 2M) carry x2 with the scale byte of beta (row concatenation, Sec. 3.9; the scale
// operand is per lane, so the two halves can use different scales); the epilogue adds output rows
// m and M + m.  Halves the matrix instructions, which at 4 bits per weight are as expensive as
// the weight stream itself.
// EXPORT (SELF only): workgroup 0 also writes the ABI-format codes for the observation points; a
// separate instantiation because that path keeps 64 code registers alive.
// SEG (FAST, canonical weights): the four loads of a super-step fetch the 256 bytes of a weight row per 16 lanes
// (four rows per instruction) instead of 64 bytes of each of 16 rows, and the wave turns them into operand order
// through 4 KB of LDS of its own (chunk c of row r at position c ^ r; no barrier), as in gemm_w4_rows_kernel.
template <int WAVES, int U, int RT, bool SELF, bool FAST, bool STACK, bool EXPORT = false, bool SEG = false>
__device__ __forceinline__ void gemm_w4_skinny_body(const GemmW4Args& a, const int64_t n0, const int64_t m0) {
  static_assert(!STACK || RT == 1, "stacked components use a single row fragment");
  static_assert(!SEG || FAST, "row segments need whole super-steps");
  constexpr bool CONTIG = true;
  __shared__ float s_part[WAVES][RT][4][64];
  __shared__ __attribute__((aligned(16))) uint8_t s_seg[SEG ? WAVES * 4096 : 16];
  extern __shared__ __attribute__((aligned(16))) uint8_t s_dyn[];  // SELF: per wave [2][M][bpw][24 B] + [M][bpw]
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int row = lane & 15, g = lane >> 4;
  const int64_t M = a.M, N = a.N, KB = a.K / 32;
  const int64_t supers = (KB + 15) / 16;  // super-steps of 16 blocks (512 k)
  const int64_t per = (supers + WAVES - 1) / WAVES;
  const int64_t s0 = min((int64_t)wave * per, supers), s1 = min(supers, s0 + per);
  constexpr bool fast = FAST;
  const int64_t wrow = min(n0 + row, N - 1);
  // Packed weights (FAST only; layout in msd.h): the 16 channels x 4 blocks that one MFMA of this workgroup
  // multiplies are one kilobyte in lane order, the 16 x 16 scale bytes of a super-step 256 contiguous bytes.
  const bool packed = FAST && a.w_packed != 0;
  const int64_t wtiles = (N + 15) / 16;
  const uint8_t* wp = packed ? a.W + (n0 / 16) * 1024 + lane * 16 : a.W + wrow * (KB * 16);
  const uint8_t* wep = packed ? a.We + (n0 / 16) * 256 + row * 16 : a.We + wrow * KB;
  const int64_t wq = wtiles * 1024, weq = wtiles * 256;  // packed: bytes between K units / super-steps
  const v8i zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
  const v4i one16 = {0x7F7F7F7F, 0x7F7F7F7F, 0x7F7F7F7F, 0x7F7F7F7F};
  v4f acc[RT];
#pragma unroll
  for (int f = 0; f < RT; ++f) acc[f] = v4f{0.f, 0.f, 0.f, 0.f};
  // SELF: wave-private LDS for the blocks [s0*16, s1*16) of every row
  const int bpw = (int)(per * 16);  // block slots per row and wave
  uint8_t* my_q = s_dyn + (size_t)wave * ((size_t)2 * M * bpw * 24 + (size_t)M * bpw);
  uint8_t* my_e = my_q + (size_t)2 * M * bpw * 24;
  bool ready = !SELF;
  for (int64_t sb = s0; sb < (SELF ? max(s1, s0 + 1) : s1); sb += U) {
    // ---- weights of this batch: block 4u+g of super-step s for MFMA u
    v8i wb[U][4];
    int wsc[U][4];
#pragma unroll
    for (int u2 = 0; u2 < U; ++u2) {
      const int64_t s = sb + u2;
      v4i sc16 = one16;
      if (s < s1 && fast) sc16 = *reinterpret_cast<const v4i*>(wep + (packed ? s * weq : s * 16));
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int64_t bi = s * 16 + (CONTIG ? 4 * u + g : 4 * g + u);
        const bool ok = s < s1 && (FAST || bi < KB);
        wb[u2][u] = zero8;
        if (ok) {
          const uint8_t* src = wp + (packed ? (4 * s + u) * wq : bi * 16);
          if constexpr (SEG)  // rows 4 u .. 4 u + 3 of the tile, chunk lane % 16 of the super-step's 256 bytes
            src = a.W + min(n0 + 4 * u + (lane >> 4), N - 1) * (KB * 16) + s * 256 + (lane & 15) * 16;
          const v4i v = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(src));
          wb[u2][u] = v8i{v[0], v[1], v[2], v[3], 0, 0, 0, 0};
        }
        wsc[u2][u] = fast ? (CONTIG ? scale_byte(sc16, u, g) : scale_byte(sc16, g, u)) : (ok ? (int)wep[bi] : 0x7F);
      }
    }
    if (SELF && !ready) {
      // decompose this wave's blocks: block c -> (row c / nb, block c % nb), one block per lane and pass
      const int64_t b_lo = s0 * 16, b_hi = min(s1 * 16, KB);
      const int nb = (int)max((int64_t)0, b_hi - b_lo);
      const int total = (int)M * nb;
      const bool al16 = a.x_aligned != 0;
#pragma unroll 1
      for (int c = lane; c < total; c += 64) {
        const int m = c / nb, bb = c - m * nb;
        const uint16_t* xb = a.x + (int64_t)m * a.ldx + (b_lo + bb) * 32;
        uint32_t w[16];
        if (al16) {
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
        uint32_t p1[6], p2[6];
        int e;
        if constexpr (EXPORT) {
          int k1[32], k2[32];
          e = mx_block_codes(w, k1, k2, a.mv);
          pack_fp6(k1, p1, a.mv.e2m1);
          pack_fp6(k2, p2, a.mv.e2m1);
          if (blockIdx.x == 0 && a.abi_q1) {  // observation points only: ABI-format codes
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
            const int64_t gb = (int64_t)m * KB + b_lo + bb;
            reinterpret_cast<uint4*>(a.abi_q1 + gb * 16)[0] = make_uint4(c1[0], c1[1], c1[2], c1[3]);
            reinterpret_cast<uint4*>(a.abi_q2 + gb * 16)[0] = make_uint4(c2[0], c2[1], c2[2], c2[3]);
            a.abi_e8m0[gb] = (uint8_t)(e + 127);
          }
        } else {
          e = mx_block_pack_fp6(w, p1, p2, a.mv);
        }
        uint2* d1 = reinterpret_cast<uint2*>(my_q + ((size_t)m * bpw + bb) * 24);
        uint2* d2 = reinterpret_cast<uint2*>(my_q + ((size_t)(M + m) * bpw + bb) * 24);
#pragma unroll
        for (int i = 0; i < 3; ++i) {
          d1[i] = make_uint2(p1[2 * i], p1[2 * i + 1]);
          d2[i] = make_uint2(p2[2 * i], p2[2 * i + 1]);
        }
        my_e[(size_t)m * bpw + bb] = (uint8_t)(e + 127);
      }
      __builtin_amdgcn_wave_barrier();
      ready = true;
    }
    // ---- activation operands and MFMAs
#pragma unroll
    for (int u2 = 0; u2 < U; ++u2) {
      const int64_t s = sb + u2;
      if (s >= s1) continue;
      v8i wseg[SEG ? 4 : 1];
      if constexpr (SEG) {
        uint8_t* my_seg = s_seg + wave * 4096;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int r = 4 * u + (lane >> 4), c = lane & 15;
          *reinterpret_cast<v4i*>(my_seg + r * 256 + ((c ^ r) & 15) * 16) =
              v4i{wb[u2][u][0], wb[u2][u][1], wb[u2][u][2], wb[u2][u][3]};
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const v4i v = *reinterpret_cast<const v4i*>(my_seg + row * 256 + (((4 * u + g) ^ row) & 15) * 16);
          wseg[u] = v8i{v[0], v[1], v[2], v[3], 0, 0, 0, 0};
        }
        __builtin_amdgcn_wave_barrier();
      }
#pragma unroll
      for (int f = 0; f < RT; ++f) {
        // source of this lane's fragment row: activation row m, component comp
        int comp = 0;
        int64_t m = FAST ? min(m0 + 16 * f + row, M - 1) : m0 + 16 * f + row;
        bool row_ok = m < M;
        if (STACK) {
          const int r = FAST ? min(row, (int)(2 * M - 1)) : row;
          comp = r >= M ? 1 : 0;
          m = r - comp * M;
          row_ok = r < 2 * M;
        }
        v4i asc16 = one16;
        if (!SELF && fast && row_ok) asc16 = *reinterpret_cast<const v4i*>(a.e8m0 + m * KB + s * 16);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int64_t bi = s * 16 + (CONTIG ? 4 * u + g : 4 * g + u);
          const bool ok = FAST || (row_ok && bi < KB);
          v8i a1 = zero8, a2 = zero8;
          int sa = 0x7F;
          if (ok) {
            if (SELF) {
              const int64_t bl = bi - s0 * 16;
              if (STACK) {
                a1 = load_fp6_lds(my_q + ((size_t)(comp * M + m) * bpw + bl) * 24);
              } else {
                a1 = load_fp6_lds(my_q + ((size_t)m * bpw + bl) * 24);
                a2 = load_fp6_lds(my_q + ((size_t)(M + m) * bpw + bl) * 24);
              }
              sa = my_e[(size_t)m * bpw + bl];
            } else {
              if (STACK) {
                a1 = load_fp6_slot((comp ? a.q2 : a.q1) + (m * KB + bi) * 8);
              } else {
                a1 = load_fp6_slot(a.q1 + (m * KB + bi) * 8);
                a2 = load_fp6_slot(a.q2 + (m * KB + bi) * 8);
              }
              sa = fast ? (CONTIG ? scale_byte(asc16, u, g) : scale_byte(asc16, g, u)) : (int)a.e8m0[m * KB + bi];
            }
          }
          const v8i wop = SEG ? wseg[SEG ? u : 0] : wb[u2][u];
          if (STACK) {
            acc[f] = mfma_scaled(a1, wop, acc[f], sa - a.mv.shift * comp, wsc[u2][u]);  // beta = alpha / 2^shift
          } else {
            acc[f] = mfma_scaled(a1, wop, acc[f], sa, wsc[u2][u]);
            acc[f] = mfma_scaled(a2, wop, acc[f], sa - a.mv.shift, wsc[u2][u]);  // beta = alpha / 2^shift
          }
        }
      }
    }
  }
#pragma unroll
  for (int f = 0; f < RT; ++f)
#pragma unroll
    for (int r = 0; r < 4; ++r) s_part[wave][f][r][lane] = acc[f][r];
  __syncthreads();
  // D[i][j]: fragment i/16, register (i%16)%4, lane ((i%16)/4)*16 + j
  for (int t = threadIdx.x; t < RT * 256; t += WAVES * 64) {
    const int i = t >> 4, j = t & 15;
    const int64_t m = m0 + i, n = n0 + j;
    if (m >= M || n >= N) continue;
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) v += s_part[w][i >> 4][i & 3][((i & 15) >> 2) * 16 + j];
    if (STACK) {  // second component: fragment row M + i (same fp32 order for every wave)
      const int i2 = (int)M + i;
      float v2 = 0.f;
#pragma unroll
      for (int w = 0; w < WAVES; ++w) v2 += s_part[w][0][i2 & 3][(i2 >> 2) * 16 + j];
      v += v2;
    }
    if (a.out_bf16)
      reinterpret_cast<uint16_t*>(a.y)[m * a.ldy + n] = f32_to_bf16_bits(v);
    else
      reinterpret_cast<float*>(a.y)[m * a.ldy + n] = v;
  }
}

template <int WAVES, int U, int RT, bool SELF, bool FAST, bool STACK, bool EXPORT = false>
__global__ __launch_bounds__(WAVES * 64) void gemm_w4_skinny_kernel(GemmW4Args a) {
  gemm_w4_skinny_body<WAVES, U, RT, SELF, FAST, STACK, EXPORT>(a, (int64_t)blockIdx.x * 16,
                                                               (int64_t)blockIdx.y * 16 * RT);
}

// Grouped form for mixture-of-experts layers (paper Sec. 7.5; rows sorted by expert, expert
// e = blockIdx.y owns rows [offs[e], offs[e+1]) and its own weights and scales).  The workgroup reads
// its expert's row range on the device and runs the stacked-component body on chunks of 8 rows.
template <int WAVES, int U, bool FAST>
__global__ __launch_bounds__(WAVES * 64) void gemm_w4_grouped_kernel(GemmW4Args a, const int32_t* __restrict__ offs) {
  const int e = blockIdx.y;
  // a.M is the total number of rows: offsets outside [0, M] (a malformed routing table) are clamped, so
  // that no row index leaves the activation and output arrays
  const int64_t r1 = min((int64_t)offs[e + 1], a.M), r0 = max((int64_t)offs[e], (int64_t)0);
  const int64_t KB = a.K / 32;
  for (int64_t c0 = r0; c0 < r1; c0 += 8) {
    GemmW4Args b = a;
    b.q1 = a.q1 + c0 * KB * 8;
    b.q2 = a.q2 + c0 * KB * 8;
    b.e8m0 = a.e8m0 + c0 * KB;
    b.W = a.W + (int64_t)e * a.N * (KB * 16);
    b.We = a.We + (int64_t)e * a.N * KB;
    b.y = a.out_bf16 ? (void*)(reinterpret_cast<uint16_t*>(a.y) + c0 * a.ldy)
                     : (void*)(reinterpret_cast<float*>(a.y) + c0 * a.ldy);
    b.M = min((int64_t)8, r1 - c0);
    gemm_w4_skinny_body<WAVES, U, 1, false, FAST, true, false, FAST>(b, (int64_t)blockIdx.x * 16, 0);
    __syncthreads();  // the wave partials in LDS are rewritten by the next chunk
  }
}

bool gemm_w4_is_fused(int64_t M, int64_t K, int64_t) { return M <= 1 && K > 0 && K <= 32768; }

// ------------------------------------------------------------------ one or two rows on packed weights, one launch
// One workgroup per CU and round: each of its waves owns one 16-channel tile over the whole K range, so the
// activation rows are decomposed once per workgroup (Alg. 2; one 32-element block per thread and pass, into LDS)
// instead of once per 16 channels, and that fits under the waves' first weight loads: kRowsDepth batches of
// kRowsU super-steps (24 KB per wave) are requested before the decomposition starts, the thread's first x block
// before those.  No separate decomposition launch, nothing materialised in HBM.
// The result is bit-identical to the kernel above: the K range is accumulated in the same four contiguous parts
// (the K ranges of that kernel's four waves), which are then added in the same order, and the two components
// travel in the same stacked rows.
constexpr int kRowsMaxWaves = 8;
constexpr int kRowsU = 2;      // super-steps (512 k) per batch
constexpr int kRowsDepth = 3;  // batches in flight per wave
constexpr int kRowsMaxM = 2;  // (8192 x 28672: 29.7 -> 26.2 us at one row, 30.6 -> 29.8 at two; 31.6 -> 33.6 at three: the
                               // decomposition before the first MFMA grows with the rows)
constexpr size_t kRowsMaxLds = 144 * 1024;

// NPRE: x blocks a thread requests before its weight batches (loads complete in order: an x block requested after
// them would wait for all of them)
// PACKED = false: the canonical layout W [N][K/2], We [N][K/32].  A B-operand load straight from it would touch 16
// weight rows with 64 bytes each per instruction; instead a wave fetches 256 contiguous bytes of a row (4 rows per
// instruction, four instructions per super-step of its 16 channels) and turns them into operand order through a
// private 8 KB of LDS: 16-byte chunk c of row r is stored at chunk position c ^ r, so that both the stores (eight
// consecutive lanes = one row's line) and the operand reads (sixteen rows at one chunk) are conflict-free.
template <int NPRE, bool PACKED>
__global__ __launch_bounds__(kRowsMaxWaves * 64) void gemm_w4_rows_kernel(GemmW4Args a, int tpw) {
  // [2M][KB][24 B] | [M][KB] | [waves][4][64] f32 | canonical weights: [waves][kRowsU][16 rows][256 B]
  extern __shared__ __attribute__((aligned(16))) uint8_t s_rows[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row = lane & 15, g = lane >> 4;
  const int M = (int)a.M;
  const int64_t N = a.N, KB = a.K / 32, supers = KB / 16;
  const int64_t wtiles = (N + 15) / 16;
  const int64_t tile_raw = (int64_t)blockIdx.x * tpw + wave;
  const int64_t tile = min(tile_raw, wtiles - 1);  // past the end: repeats the last tile, nothing stored
  uint8_t* sA = s_rows;
  uint8_t* sE = sA + (size_t)2 * M * KB * 24;
  float* s_fin = reinterpret_cast<float*>(sE + (((size_t)M * KB + 15) & ~(size_t)15)) + wave * 256;
  const int nblocks = M * (int)KB;
  const bool al16 = a.x_aligned != 0;
  auto load_x = [&](int c, uint32_t (&w)[16]) {
    const int m = c / (int)KB, bb = c - m * (int)KB;
    const uint16_t* xb = a.x + (int64_t)m * a.ldx + (int64_t)bb * 32;
    if (al16) {
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
  };
  auto decompose = [&](int c, const uint32_t (&w)[16]) {
    const int m = c / (int)KB, bb = c - m * (int)KB;
    uint32_t p1[6], p2[6];
    const int e = mx_block_pack_fp6(w, p1, p2, a.mv);
    uint2* d1 = reinterpret_cast<uint2*>(sA + ((size_t)m * KB + bb) * 24);
    uint2* d2 = reinterpret_cast<uint2*>(sA + ((size_t)(M + m) * KB + bb) * 24);
#pragma unroll
    for (int i = 0; i < 3; ++i) {
      d1[i] = make_uint2(p1[2 * i], p1[2 * i + 1]);
      d2[i] = make_uint2(p2[2 * i], p2[2 * i + 1]);
    }
    sE[(size_t)m * KB + bb] = (uint8_t)(e + 127);
  };
  // ---- this thread's first x block, then the first weight batches, then the decomposition
  uint32_t w0[NPRE][16];
#pragma unroll
  for (int i = 0; i < NPRE; ++i) load_x(min(tid + i * (int)blockDim.x, nblocks - 1), w0[i]);
  const int64_t wq = wtiles * 1024, weq = wtiles * 256;  // packed: bytes between K units / super-steps
  // canonical: instruction u of a super-step covers the 256 bytes of rows 4 u .. 4 u + 3
  int64_t crow[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) crow[u] = min(tile * 16 + 4 * u + (lane >> 4), N - 1) * (KB * 16);
  const uint8_t* wp = PACKED ? a.W + tile * 1024 + lane * 16 : a.W + 16 * (lane & 15);
  const uint8_t* wep = PACKED ? a.We + tile * 256 + row * 16 : a.We + min(tile * 16 + row, N - 1) * KB;
  uint8_t* stage = reinterpret_cast<uint8_t*>(reinterpret_cast<float*>(sE + (((size_t)M * KB + 15) & ~(size_t)15)) +
                                              (size_t)blockDim.x / 64 * 256) + (size_t)wave * (kRowsU * 4096);
  struct Batch {
    v4i w[kRowsU][4], sc[kRowsU];
  };
  auto load_w = [&](int64_t b, Batch& t) {  // batches past the end repeat the last super-step (never multiplied)
#pragma unroll
    for (int u2 = 0; u2 < kRowsU; ++u2) {
      const int64_t sp = min(b * kRowsU + u2, supers - 1);
      t.sc[u2] = *reinterpret_cast<const v4i*>(wep + (PACKED ? sp * weq : sp * 16));
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint8_t* src = PACKED ? wp + (4 * sp + u) * wq : wp + crow[u] + sp * 256;
        t.w[u2][u] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(src));
      }
    }
  };
  Batch B0, B1, B2;
  static_assert(kRowsDepth == 3, "three rotating batches are written out below");
  load_w(0, B0);
  load_w(1, B1);
  load_w(2, B2);
#pragma unroll
  for (int i = 0; i < NPRE; ++i)
    if (tid + i * (int)blockDim.x < nblocks) decompose(tid + i * (int)blockDim.x, w0[i]);
#pragma unroll 1
  for (int c = tid + NPRE * blockDim.x; c < nblocks; c += blockDim.x) {
    uint32_t w[16];
    load_x(c, w);
    decompose(c, w);
  }
  // the operands are in LDS; a plain __syncthreads() would also wait for the weight batches in flight
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  // ---- K loop: four contiguous parts, each its own accumulator
  const int64_t per = (supers + 3) / 4;
  const v4f zero4 = {0.f, 0.f, 0.f, 0.f};
  v4f part[4] = {zero4, zero4, zero4, zero4};
  const int r = min(row, 2 * M - 1);  // stacked fragment row: [0, M) first component, [M, 2M) residual
  const int comp = r >= M ? 1 : 0, m = r - comp * M;
  const uint8_t* arow = sA + (size_t)r * KB * 24;
  const uint8_t* erow = sE + (size_t)m * KB;
  const int shift = a.mv.shift * comp;  // beta = alpha / 2^shift
  auto multiply = [&](int64_t b, const Batch& t) {
    if constexpr (!PACKED) {
      // the batch's lines into operand order: row r = 4 u + lane / 16, chunk c = lane % 16
#pragma unroll
      for (int u2 = 0; u2 < kRowsU; ++u2)
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int r4 = 4 * u + (lane >> 4), c = lane & 15;
          *reinterpret_cast<v4i*>(stage + u2 * 4096 + r4 * 256 + ((c ^ r4) & 15) * 16) = t.w[u2][u];
        }
      __builtin_amdgcn_wave_barrier();
    }
#pragma unroll
    for (int u2 = 0; u2 < kRowsU; ++u2) {
      const int64_t sp = b * kRowsU + u2;
      if (sp < supers) {
        const int q = (int)(sp / per);
        v4f acc = q == 0 ? part[0] : q == 1 ? part[1] : q == 2 ? part[2] : part[3];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int64_t bi = sp * 16 + 4 * u + g;
          const v8i a1 = load_fp6_lds(arow + bi * 24);
          const int sa = (int)erow[bi] - shift;
          v4i wv = t.w[u2][u];
          if constexpr (!PACKED)
            wv = *reinterpret_cast<const v4i*>(stage + u2 * 4096 + row * 256 + (((4 * u + g) ^ row) & 15) * 16);
          const v8i wb = {wv[0], wv[1], wv[2], wv[3], 0, 0, 0, 0};
          acc = mfma_scaled(a1, wb, acc, sa, scale_byte(t.sc[u2], u, g));
        }
#pragma unroll
        for (int qq = 0; qq < 4; ++qq)
          if (qq == q) part[qq] = acc;
      }
    }
  };
  const int64_t nb = (supers + kRowsU - 1) / kRowsU;
  for (int64_t b = 0; b < nb; b += kRowsDepth) {
    multiply(b, B0);
    load_w(b + 3, B0);
    multiply(b + 1, B1);
    load_w(b + 4, B1);
    multiply(b + 2, B2);
    load_w(b + 5, B2);
  }
  // ---- the four parts in order, then the two components: D[i][j] sits in register i % 4 of lane (i / 4) * 16 + j
  v4f fin;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float v = 0.f;
#pragma unroll
    for (int qq = 0; qq < 4; ++qq) v += part[qq][i];
    fin[i] = v;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) s_fin[i * 64 + lane] = fin[i];
  __builtin_amdgcn_wave_barrier();
  if (tile_raw < wtiles) {
    for (int t = lane; t < M * 16; t += 64) {
      const int mm = t >> 4, j = t & 15, i2 = M + mm;
      const float v = s_fin[(mm & 3) * 64 + (mm >> 2) * 16 + j] + s_fin[(i2 & 3) * 64 + (i2 >> 2) * 16 + j];
      const int64_t n = tile * 16 + j;
      if (n < N) {
        if (a.out_bf16)
          reinterpret_cast<uint16_t*>(a.y)[(int64_t)mm * a.ldy + n] = f32_to_bf16_bits(v);
        else
          reinterpret_cast<float*>(a.y)[(int64_t)mm * a.ldy + n] = v;
      }
    }
  }
}

// tiles per workgroup: the 16-channel tiles dealt evenly to 256 CUs per round, at most eight (one per wave)
static int w4_rows_tpw(int64_t N) {
  const int64_t tiles = cdiv(N, 16);
  const int64_t rounds = cdiv(tiles, (int64_t)kRowsMaxWaves * 256);
  return (int)cdiv(tiles, 256 * rounds);
}
static size_t w4_rows_lds(int64_t M, int64_t K, int tpw, bool packed) {
  const size_t KB = (size_t)K / 32;
  return 2 * (size_t)M * KB * 24 + align_up((size_t)M * KB, 16) + (size_t)tpw * 1024 +
         (packed ? 0 : (size_t)tpw * kRowsU * 4096);
}
bool gemm_w4_rows_applies(int64_t M, int64_t K, int64_t N, bool scales_aligned) {
  if (M < 1 || M > kRowsMaxM || K < 512 || K % 512 != 0 || !scales_aligned) return false;
  const int tpw = w4_rows_tpw(N);
  // with few tiles per CU the waves of the K-split kernel pull more data at once
  return tpw >= 4 && w4_rows_lds(M, K, tpw, false) <= kRowsMaxLds;
}
int launch_gemm_w4_rows(const GemmW4Args& a, hipStream_t stream) {
  if (a.x == nullptr || !gemm_w4_rows_applies(a.M, a.K, a.N, a.scales_aligned != 0)) return MSD_ERR_INVALID_ARG;
  const int tpw = w4_rows_tpw(a.N);
  const size_t lds = w4_rows_lds(a.M, a.K, tpw, a.w_packed != 0);
  static bool attr_set = false;
  if (!attr_set) {
    MSD_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_w4_rows_kernel<2, true>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)kRowsMaxLds));
    MSD_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_w4_rows_kernel<2, false>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)kRowsMaxLds));
    attr_set = true;
  }
  const dim3 grid((unsigned)cdiv(cdiv(a.N, 16), tpw)), block(tpw * 64);
  // two x blocks per thread requested up front (with fewer the second request repeats the last block; an instance
  // with one spilled); long rows take further passes after the weight batches
  if (a.w_packed)
    hipLaunchKernelGGL((gemm_w4_rows_kernel<2, true>), grid, block, lds, stream, a, tpw);
  else
    hipLaunchKernelGGL((gemm_w4_rows_kernel<2, false>), grid, block, lds, stream, a, tpw);
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}


template <int WAVES, int U, int RT, bool SELF, bool STACK = false>
static int launch_w4(const GemmW4Args& a, hipStream_t stream) {
  size_t dyn = 0;
  if (SELF) {
    const int64_t supers = (a.K / 32 + 15) / 16;
    const int64_t bpw = cdiv(supers, WAVES) * 16;
    dyn = (size_t)WAVES * (2 * a.M * bpw * 24 + a.M * bpw);
    dyn = align_up(dyn, 16);
  }
  const dim3 grid((unsigned)cdiv(a.N, 16), (unsigned)cdiv(a.M, 16 * RT));
  const bool fast = (a.K / 32) % 16 == 0 && a.scales_aligned;
  if (SELF && a.abi_q1) {  // observation points requested
    if (fast)
      hipLaunchKernelGGL((gemm_w4_skinny_kernel<WAVES, U, RT, SELF, true, STACK, SELF>), grid, dim3(WAVES * 64), dyn, stream, a);
    else
      hipLaunchKernelGGL((gemm_w4_skinny_kernel<WAVES, U, RT, SELF, false, STACK, SELF>), grid, dim3(WAVES * 64), dyn, stream, a);
  } else if (fast) {
    hipLaunchKernelGGL((gemm_w4_skinny_kernel<WAVES, U, RT, SELF, true, STACK>), grid, dim3(WAVES * 64), dyn, stream, a);
  } else {
    hipLaunchKernelGGL((gemm_w4_skinny_kernel<WAVES, U, RT, SELF, false, STACK>), grid, dim3(WAVES * 64), dyn, stream, a);
  }
  return MSD_OK;
}

// ------------------------------------------------------------------ tiled (observation points, or K not a multiple of 64 / 512)
// v_mfma_scale_f32_32x32x64_f8f6f4: lane l holds row/column l%32 and K block l/32 (two blocks
// per instruction).  Workgroup tile BM x BN, K stage of 4 blocks (128 k), LDS double buffering
// with register staging of the next stage.  LDS operand layout is [block][row][24 B] for the
// FP6 components and [block][column][16 B] for the FP4 weights, i.e. exactly lane order, so all
// fragment reads are linear and conflict-free.  Both components accumulate into one fp32
// accumulator; beta's scale byte is alpha's minus 4.
__device__ __forceinline__ v16f mfma32_scaled(v8i a, v8i b, v16f c, int sa, int sb) {
  return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 2, 4, 0, sa, 0, sb);
}

constexpr int kW4GroupM = 8;

template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(WM * WN * 64) void gemm_w4_tiled_kernel(GemmW4Args a, int tiles_m, int tiles_n) {
  constexpr int THREADS = WM * WN * 64;
  constexpr int TM = BM / WM, TN = BN / WN, FM = TM / 32, FN = TN / 32;
  constexpr int A_ITEMS = BM * 4 * 2, B_ITEMS = BN * 4;
  constexpr int LA = (A_ITEMS + THREADS - 1) / THREADS, LB = (B_ITEMS + THREADS - 1) / THREADS;
  constexpr int SZ_A = 4 * BM * 24, SZ_B = 4 * BN * 16, SZ_AE = BM * 4, SZ_BE = BN * 4;
  constexpr int STAGE = 2 * SZ_A + SZ_B + SZ_AE + SZ_BE;
  extern __shared__ __attribute__((aligned(16))) uint8_t smem4[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int l32 = lane & 31, kb = lane >> 5;
  const int64_t M = a.M, N = a.N, KB = a.K / 32;
  const int total = tiles_m * tiles_n;
  int id = blockIdx.x;
  {
    const int per_xcd = (total + 7) / 8;
    id = (id % 8) * per_xcd + id / 8;
  }
  if (id >= total) return;
  const int group = id / (kW4GroupM * tiles_n);
  const int first_m = group * kW4GroupM;
  const int rows_in_group = min(kW4GroupM, tiles_m - first_m);
  const int in_group = id - group * kW4GroupM * tiles_n;
  const int tm = first_m + in_group % rows_in_group;
  const int tn = in_group / rows_in_group;
  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;
  const bool dword_scales = (KB % 4) == 0 && a.scales_aligned;
  const v8i zero8 = {0, 0, 0, 0, 0, 0, 0, 0};

  // ---- staging registers for one stage
  uint4 ra_lo[LA];
  uint2 ra_hi[LA];
  uint4 rb[LB];
  uint32_t rae = 0x7F7F7F7Fu, rbe = 0x7F7F7F7Fu, rbe2 = 0x7F7F7F7Fu;
  auto gload = [&](int kt) {
    const int64_t b0 = (int64_t)kt * 4;
#pragma unroll
    for (int i = 0; i < LA; ++i) {
      const int idx = tid + i * THREADS;
      ra_lo[i] = make_uint4(0, 0, 0, 0);
      ra_hi[i] = make_uint2(0, 0);
      if (idx < A_ITEMS) {
        const int comp = idx / (BM * 4), rem = idx - comp * (BM * 4);
        const int r = rem >> 2, blk = rem & 3;
        const int64_t m = min(m0 + r, M - 1);
        if (b0 + blk < KB) {
          const uint32_t* p = (comp ? a.q2 : a.q1) + (m * KB + b0 + blk) * 8;
          ra_lo[i] = *reinterpret_cast<const uint4*>(p);
          ra_hi[i] = *reinterpret_cast<const uint2*>(p + 4);
        }
      }
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
      const int idx = tid + i * THREADS;
      rb[i] = make_uint4(0, 0, 0, 0);
      if (idx < B_ITEMS) {
        const int c = idx >> 2, blk = idx & 3;
        const int64_t n = min(n0 + c, N - 1);
        if (b0 + blk < KB) {
          const v4i v = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(a.W + n * (KB * 16) + (b0 + blk) * 16));
          rb[i] = make_uint4((uint32_t)v[0], (uint32_t)v[1], (uint32_t)v[2], (uint32_t)v[3]);
        }
      }
    }
    rae = rbe = rbe2 = 0x7F7F7F7Fu;
    if (tid < BM) {
      const int64_t m = min(m0 + tid, M - 1);
      const uint8_t* pe = a.e8m0 + m * KB + b0;
      if (dword_scales) {
        rae = *reinterpret_cast<const uint32_t*>(pe);
      } else {
        uint32_t v = 0;
#pragma unroll
        for (int u = 0; u < 4; ++u) v |= (uint32_t)(b0 + u < KB ? pe[u] : 0x7F) << (8 * u);
        rae = v;
      }
    }
    for (int c = tid; c < BN; c += THREADS) {  // BN <= 2*THREADS: at most two passes, kept simple
      const int64_t n = min(n0 + c, N - 1);
      const uint8_t* pe = a.We + n * KB + b0;
      uint32_t v = 0;
      if (dword_scales) {
        v = *reinterpret_cast<const uint32_t*>(pe);
      } else {
#pragma unroll
        for (int u = 0; u < 4; ++u) v |= (uint32_t)(b0 + u < KB ? pe[u] : 0x7F) << (8 * u);
      }
      if (c == tid) rbe = v; else rbe2 = v;
    }
  };
  auto sstore = [&](int buf) {
    uint8_t* st = smem4 + buf * STAGE;
#pragma unroll
    for (int i = 0; i < LA; ++i) {
      const int idx = tid + i * THREADS;
      if (idx < A_ITEMS) {
        const int comp = idx / (BM * 4), rem = idx - comp * (BM * 4);
        const int r = rem >> 2, blk = rem & 3;
        uint2* d = reinterpret_cast<uint2*>(st + comp * SZ_A + (blk * BM + r) * 24);
        d[0] = make_uint2(ra_lo[i].x, ra_lo[i].y);
        d[1] = make_uint2(ra_lo[i].z, ra_lo[i].w);
        d[2] = ra_hi[i];
      }
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
      const int idx = tid + i * THREADS;
      if (idx < B_ITEMS) {
        const int c = idx >> 2, blk = idx & 3;
        *reinterpret_cast<uint4*>(st + 2 * SZ_A + (blk * BN + c) * 16) = rb[i];
      }
    }
    if (tid < BM) *reinterpret_cast<uint32_t*>(st + 2 * SZ_A + SZ_B + tid * 4) = rae;
    if (tid < BN) *reinterpret_cast<uint32_t*>(st + 2 * SZ_A + SZ_B + SZ_AE + tid * 4) = rbe;
    if (tid + THREADS < BN) *reinterpret_cast<uint32_t*>(st + 2 * SZ_A + SZ_B + SZ_AE + (tid + THREADS) * 4) = rbe2;
  };

  v16f acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int KT = (int)((KB + 3) / 4);
  if (KT > 0) {
    gload(0);
    sstore(0);
  }
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < KT) gload(kt + 1);
    const uint8_t* st = smem4 + buf * STAGE;
#pragma unroll
    for (int kp = 0; kp < 2; ++kp) {
      const int blk = kp * 2 + kb;
      v8i fb[FN];
      int sb[FN];
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        const int c = wn * TN + 32 * j + l32;
        const uint4 v = *reinterpret_cast<const uint4*>(st + 2 * SZ_A + (blk * BN + c) * 16);
        fb[j] = v8i{(int)v.x, (int)v.y, (int)v.z, (int)v.w, 0, 0, 0, 0};
        sb[j] = st[2 * SZ_A + SZ_B + SZ_AE + c * 4 + blk];
      }
#pragma unroll
      for (int i = 0; i < FM; ++i) {
        const int r = wm * TM + 32 * i + l32;
        const v8i f1 = load_fp6_lds(st + (blk * BM + r) * 24);
        const v8i f2 = load_fp6_lds(st + SZ_A + (blk * BM + r) * 24);
        const int sa = st[2 * SZ_A + SZ_B + r * 4 + blk];
#pragma unroll
        for (int j = 0; j < FN; ++j) {
          acc[i][j] = mfma32_scaled(f1, fb[j], acc[i][j], sa, sb[j]);
          acc[i][j] = mfma32_scaled(f2, fb[j], acc[i][j], sa - a.mv.shift, sb[j]);
        }
      }
    }
    if (kt + 1 < KT) sstore(buf ^ 1);
    __syncthreads();
  }
  (void)zero8;
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int64_t m = m0 + wm * TM + 32 * i + (r >> 2) * 8 + kb * 4 + (r & 3);
      if (m >= M) continue;
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        const int64_t n = n0 + wn * TN + 32 * j + l32;
        if (n >= N) continue;
        if (a.out_bf16)
          reinterpret_cast<uint16_t*>(a.y)[m * a.ldy + n] = f32_to_bf16_bits(acc[i][j][r]);
        else
          reinterpret_cast<float*>(a.y)[m * a.ldy + n] = acc[i][j][r];
      }
    }
}

template <int BM, int BN, int WM, int WN>
static int launch_w4_tiled(const GemmW4Args& a, hipStream_t stream) {
  const int tiles_m = (int)cdiv(a.M, BM), tiles_n = (int)cdiv(a.N, BN);
  const int total = tiles_m * tiles_n;
  const int grid = ((total + 7) / 8) * 8;
  const size_t lds = (size_t)2 * (2 * 4 * BM * 24 + 4 * BN * 16 + BM * 4 + BN * 4);
  static bool attr_set = false;
  if (!attr_set && lds > 64 * 1024) {
    MSD_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_w4_tiled_kernel<BM, BN, WM, WN>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_set = true;
  }
  hipLaunchKernelGGL((gemm_w4_tiled_kernel<BM, BN, WM, WN>), dim3(grid), dim3(WM * WN * 64), lds, stream, a, tiles_m,
                     tiles_n);
  return MSD_OK;
}

int launch_gemm_w4_grouped(const GemmW4Args& a, const int32_t* offs, int E, hipStream_t stream) {
  if (E <= 0 || a.N == 0) return MSD_OK;
  const dim3 grid((unsigned)cdiv(a.N, 16), (unsigned)E);
  const bool fast = (a.K / 32) % 16 == 0 && a.scales_aligned;
  if (fast)
    hipLaunchKernelGGL((gemm_w4_grouped_kernel<4, 2, true>), grid, dim3(4 * 64), 0, stream, a, offs);
  else
    hipLaunchKernelGGL((gemm_w4_grouped_kernel<4, 2, false>), grid, dim3(4 * 64), 0, stream, a, offs);
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

// ------------------------------------------------------------------ one-time weight repack (msd_pack_weights_w4)
// codes: one thread per 16-byte block of a channel; scales: one thread per (super-step, channel)
__global__ __launch_bounds__(256) void pack_weights_w4_kernel(const uint8_t* __restrict__ W, const uint8_t* __restrict__ We,
                                                              int64_t N, int64_t KB, uint8_t* __restrict__ Wp,
                                                              uint8_t* __restrict__ Ep) {
  const int64_t tiles = (N + 15) / 16;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t pieces = (KB / 4) * tiles * 64;
  if (gid < pieces) {
    const int lane = (int)(gid & 63), r = lane & 15, g = lane >> 4;
    const int64_t tile = (gid >> 6) % tiles, q = (gid >> 6) / tiles;
    const int64_t n = tile * 16 + r;
    v4i v = {0, 0, 0, 0};
    if (n < N) v = *reinterpret_cast<const v4i*>(W + (n * KB + 4 * q + g) * 16);
    *reinterpret_cast<v4i*>(Wp + gid * 16) = v;
  }
  const int64_t recs = (KB / 16) * tiles * 16;
  if (gid < recs) {
    const int r = (int)(gid & 15);
    const int64_t tile = (gid >> 4) % tiles, s = (gid >> 4) / tiles;
    const int64_t n = tile * 16 + r;
    uint8_t b[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) b[i] = n < N ? We[n * KB + s * 16 + i] : (uint8_t)0x7F;
#pragma unroll
    for (int i = 0; i < 16; ++i) Ep[gid * 16 + i] = b[i];
  }
}

int launch_pack_weights_w4(const uint8_t* W, const uint8_t* We, int64_t N, int64_t K, uint8_t* Wp, uint8_t* Ep,
                           hipStream_t stream) {
  const int64_t KB = K / 32, tiles = (N + 15) / 16;
  const int64_t pieces = (KB / 4) * tiles * 64;
  hipLaunchKernelGGL(pack_weights_w4_kernel, dim3((unsigned)cdiv(pieces, 256)), dim3(256), 0, stream, W, We, N, KB, Wp, Ep);
  MSD_LAUNCH_CHECK();
  // second part of the scale array: the same bytes in the stage order of the many-row kernel, so that no call has to
  // rearrange them
  return launch_transpose_w_scales(We, N, K, Ep + w4_packed_scales_decode_bytes(N, K), stream);
}

int launch_gemm_w4(const GemmW4Args& a, hipStream_t stream) {
  if (a.M == 0 || a.N == 0) return MSD_OK;
  // packed weights: the register-operand kernel in its unpredicated form only
  if (a.w_packed && (a.M > 16 || (a.K / 32) % 16 != 0)) return MSD_ERR_UNSUPPORTED;
  int rc;
  if (a.x != nullptr) {  // single launch (gemm_w4_is_fused)
    rc = launch_w4<4, 2, 1, true, true>(a, stream);
  } else if (a.M <= 8) {
    rc = launch_w4<4, 2, 1, false, true>(a, stream);  // both components in one row fragment
  } else if (a.M <= 16) {
    rc = launch_w4<4, 2, 1, false>(a, stream);
  } else if (a.M <= 32) {
    rc = launch_w4_tiled<32, 128, 1, 4>(a, stream);
  } else {
    // more than 32 rows with K not a multiple of 64, or observation points requested (otherwise
    // the many-row pipeline of gemm_w4_prefill.hip runs)
    rc = launch_w4_tiled<128, 256, 2, 2>(a, stream);
  }
  if (rc) return rc;
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

}  // namespace msd
