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
// agree: over a super-step of 16 blocks, lane group g = l/16 takes blocks 4g..4g+3, so each
// lane reads 64 contiguous bytes of W and one dword of four scale bytes, and MFMA u
// (u = 0..3) consumes block 4g+u with scale byte u selected by op_sel.
#include "kernels.hpp"

namespace msd {

template <int SEL>
__device__ __forceinline__ v4f mfma_scaled(v8i a, v8i b, v4f c, int sa, int sb) {
  // A: FP6 E2M3 (cbsz = 2), B: FP4 E2M1 (blgp = 4); scale byte SEL of sa / sb
  return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 2, 4, SEL, sa, SEL, sb);
}

struct ABlock4 {  // four consecutive FP6 blocks of one row (6 dwords each) and their scale bytes
  v8i blk[4];
  int scale;
};

// rows [m0, m0+16): lane (row = l%16, g = l/16) loads blocks [b0 + 4g, +4) of row m0+row
__device__ __forceinline__ void load_a(const uint32_t* __restrict__ q, const uint8_t* __restrict__ e,
                                       int64_t M, int64_t KB, int64_t m, int64_t b, bool fast,
                                       ABlock4& out) {
  const v8i zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int u = 0; u < 4; ++u) out.blk[u] = zero;
  out.scale = 0x7F7F7F7F;
  if (m >= M) return;
  const uint32_t* p = q + (m * KB + b) * 8;
  const uint8_t* pe = e + m * KB + b;
  if (fast) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint4 lo = *reinterpret_cast<const uint4*>(p + 8 * u);
      const uint2 hi = *reinterpret_cast<const uint2*>(p + 8 * u + 4);
      out.blk[u] = v8i{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, 0, 0};
    }
    out.scale = *reinterpret_cast<const int*>(pe);
  } else {
    uint32_t sc = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      uint32_t byte = 0x7F;
      if (b + u < KB) {
        const uint4 lo = *reinterpret_cast<const uint4*>(p + 8 * u);
        const uint2 hi = *reinterpret_cast<const uint2*>(p + 8 * u + 4);
        out.blk[u] = v8i{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, 0, 0};
        byte = pe[u];
      }
      sc |= byte << (8 * u);
    }
    out.scale = (int)sc;
  }
}

// One workgroup: rows [m0, m0 + 16*RT) x 16 output channels; WAVES waves split K.
template <int WAVES, int RT>
__global__ __launch_bounds__(WAVES * 64) void gemm_w4_skinny_kernel(GemmW4Args a) {
  __shared__ float s_part[WAVES][RT][4][64];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int row = lane & 15, g = lane >> 4;
  const int64_t M = a.M, N = a.N, KB = a.K / 32;
  const int64_t n0 = (int64_t)blockIdx.x * 16;
  const int64_t m0 = (int64_t)blockIdx.y * 16 * RT;
  const int64_t supers = (KB + 15) / 16;  // super-steps of 16 blocks (512 k)
  const int64_t per = (supers + WAVES - 1) / WAVES;
  const int64_t s0 = wave * per, s1 = min(supers, s0 + per);
  const bool fast = (KB % 16) == 0;  // no ragged super-step, dword-aligned scale rows
  const int64_t wrow = min(n0 + row, N - 1);
  const uint8_t* wp = a.W + wrow * (KB * 16);
  const uint8_t* wep = a.We + wrow * KB;
  const v8i zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
  v4f acc[RT];
#pragma unroll
  for (int f = 0; f < RT; ++f) acc[f] = v4f{0.f, 0.f, 0.f, 0.f};
  for (int64_t s = s0; s < s1; ++s) {
    const int64_t b = s * 16 + 4 * g;  // first of this lane's four blocks
    v8i wb[4];
    int wscale;
    if (fast) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const v4i v = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(wp + (b + u) * 16));
        wb[u] = v8i{v[0], v[1], v[2], v[3], 0, 0, 0, 0};
      }
      wscale = *reinterpret_cast<const int*>(wep + b);
    } else {
      uint32_t sc = 0;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        uint32_t byte = 0x7F;
        wb[u] = zero8;
        if (b + u < KB) {
          const uint4 v = *reinterpret_cast<const uint4*>(wp + (b + u) * 16);
          wb[u] = v8i{(int)v.x, (int)v.y, (int)v.z, (int)v.w, 0, 0, 0, 0};
          byte = wep[b + u];
        }
        sc |= byte << (8 * u);
      }
      wscale = (int)sc;
    }
#pragma unroll
    for (int f = 0; f < RT; ++f) {
      ABlock4 a1, a2;
      load_a(a.q1, a.e8m0, M, KB, m0 + 16 * f + row, b, fast, a1);
      load_a(a.q2, a.e8m0, M, KB, m0 + 16 * f + row, b, fast, a2);
      const int sbeta = a2.scale - 0x04040404;  // beta = alpha / 16: every E8M0 byte minus 4
      acc[f] = mfma_scaled<0>(a1.blk[0], wb[0], acc[f], a1.scale, wscale);
      acc[f] = mfma_scaled<1>(a1.blk[1], wb[1], acc[f], a1.scale, wscale);
      acc[f] = mfma_scaled<2>(a1.blk[2], wb[2], acc[f], a1.scale, wscale);
      acc[f] = mfma_scaled<3>(a1.blk[3], wb[3], acc[f], a1.scale, wscale);
      acc[f] = mfma_scaled<0>(a2.blk[0], wb[0], acc[f], sbeta, wscale);
      acc[f] = mfma_scaled<1>(a2.blk[1], wb[1], acc[f], sbeta, wscale);
      acc[f] = mfma_scaled<2>(a2.blk[2], wb[2], acc[f], sbeta, wscale);
      acc[f] = mfma_scaled<3>(a2.blk[3], wb[3], acc[f], sbeta, wscale);
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
    if (a.out_bf16)
      reinterpret_cast<uint16_t*>(a.y)[m * a.ldy + n] = f32_to_bf16_bits(v);
    else
      reinterpret_cast<float*>(a.y)[m * a.ldy + n] = v;
  }
}

int launch_gemm_w4(const GemmW4Args& a, hipStream_t stream) {
  if (a.M == 0 || a.N == 0) return MSD_OK;
  if (a.M <= 16) {
    hipLaunchKernelGGL((gemm_w4_skinny_kernel<8, 1>), dim3((unsigned)cdiv(a.N, 16), 1), dim3(512), 0, stream, a);
  } else {
    hipLaunchKernelGGL((gemm_w4_skinny_kernel<8, 2>), dim3((unsigned)cdiv(a.N, 16), (unsigned)cdiv(a.M, 32)),
                       dim3(512), 0, stream, a);
  }
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

}  // namespace msd
