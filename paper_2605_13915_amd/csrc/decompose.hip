// Activation decomposition kernels (paper Sec. 3.2 and Sec. 3.2.1 / Alg. 2) for gfx950.
//
// INT8:   one workgroup per activation row: 16-byte loads, wave/LDS max-reduction for
//         ||x||_inf, then both quantisation passes from registers; each thread writes 16
//         codes per 16-byte store.  HBM/L2-bound: 2 B in, 2 B out per element.
// MXFP4:  one thread per 32-element block (no cross-lane reduction: the block max is the
//         only reduction and beta needs none).  Writes the ABI format (4-bit codes) and/or
//         the GEMM's internal operand format (FP6-E2M3 codes, 24 B per block in a 32 B slot).
#include "decompose_int8_dev.hpp"
#include "decompose_mxfp4_dev.hpp"
#include "kernels.hpp"

namespace msd {

// ---------------------------------------------------------------- INT8
constexpr int kDecThreads = 256;

__global__ __launch_bounds__(kDecThreads) void decompose_int8_kernel(
    const uint16_t* __restrict__ x, int64_t ldx, int K, int8_t* __restrict__ q1,
    int8_t* __restrict__ q2, int64_t ldq, float* __restrict__ alpha_out, int aligned, int64_t a_step,
    int a_bk, float num1, float num2, int frag_rt, int M) {
  __shared__ float s_red[kDecThreads / kWave];
  const int64_t m = blockIdx.x;
  if (frag_rt)  // fragment-major layout for the register-operand GEMM: q1 is the array base
    decompose_row_int8_block<kDecThreads>(x + m * ldx, K, q1, q2, alpha_out + m, aligned != 0, s_red, num1,
                                          num2, 0, m, 64, frag_rt, M);
  else if (a_step)  // blocked layout for the asynchronous-fill GEMM: q1 / q2 are the array bases
    decompose_row_int8_block<kDecThreads>(x + m * ldx, K, q1, q2, alpha_out + m, aligned != 0, s_red, num1,
                                          num2, a_step, m, a_bk);
  else
    decompose_row_int8_block<kDecThreads>(x + m * ldx, K, q1 + m * ldq, q2 + m * ldq, alpha_out + m,
                                          aligned != 0, s_red, num1, num2);
}

int launch_decompose_int8(const uint16_t* x, int64_t M, int64_t K, int64_t ldx, int8_t* q1,
                          int8_t* q2, int64_t ldq, float* alpha, int64_t a_step, int a_bk, Int8Range rg,
                          hipStream_t stream, int frag_rt) {
  if (M == 0 || K == 0) return MSD_OK;
  const int aligned = ((reinterpret_cast<uintptr_t>(x) & 15) == 0 && (ldx % 8) == 0) ? 1 : 0;
  hipLaunchKernelGGL(decompose_int8_kernel, dim3((unsigned)M), dim3(kDecThreads), 0, stream, x, ldx,
                     (int)K, q1, q2, ldq, alpha, aligned, a_step, a_bk, rg.num1, rg.num2, frag_rt, (int)M);
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

// ---------------------------------------------------------------- MXFP4
// abi_q1/abi_q2/abi_e8m0: ABI outputs (nullable).  op_q1/op_q2: FP6 operand slots, 32 B per
// block ([M][K/32][32 B], first 24 B used), op_e8m0: alpha bytes [M][K/32] (nullable group).
__global__ __launch_bounds__(256) void decompose_mxfp4_kernel(
    const uint16_t* __restrict__ x, int64_t ldx, int64_t M, int KB, uint8_t* __restrict__ abi_q1,
    uint8_t* __restrict__ abi_q2, uint8_t* __restrict__ abi_e8m0, uint32_t* __restrict__ op_q1,
    uint32_t* __restrict__ op_q2, uint8_t* __restrict__ op_e8m0, int aligned, MxVariant mv) {
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= M * KB) return;
  const int64_t m = gid / KB;
  const int b = (int)(gid % KB);
  const uint16_t* xb = x + m * ldx + (int64_t)b * 32;
  uint32_t w[16];
  if (aligned) {
    const uint4* q = reinterpret_cast<const uint4*>(xb);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      uint4 v = q[i];
      w[4 * i] = v.x; w[4 * i + 1] = v.y; w[4 * i + 2] = v.z; w[4 * i + 3] = v.w;
    }
  } else {
#pragma unroll
    for (int i = 0; i < 16; ++i) w[i] = (uint32_t)xb[2 * i] | ((uint32_t)xb[2 * i + 1] << 16);
  }
  int k1[32], k2[32];
  const int e = mx_block_codes(w, k1, k2, mv);
  const uint8_t ebyte = (uint8_t)(e + 127);
  if (abi_q1) {
    uint32_t a[4], c[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      uint32_t pa = 0, pc = 0;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        pa |= nibble4(k1[j * 8 + i]) << (4 * i);
        pc |= nibble4(k2[j * 8 + i]) << (4 * i);
      }
      a[j] = pa;
      c[j] = pc;
    }
    reinterpret_cast<uint4*>(abi_q1 + (m * KB + b) * 16)[0] = make_uint4(a[0], a[1], a[2], a[3]);
    reinterpret_cast<uint4*>(abi_q2 + (m * KB + b) * 16)[0] = make_uint4(c[0], c[1], c[2], c[3]);
    abi_e8m0[m * KB + b] = ebyte;
  }
  if (op_q1) {
    uint32_t p[6];
    pack_fp6(k1, p, mv.e2m1);
    uint32_t* d1 = op_q1 + (m * KB + b) * 8;
    reinterpret_cast<uint4*>(d1)[0] = make_uint4(p[0], p[1], p[2], p[3]);
    reinterpret_cast<uint2*>(d1)[2] = make_uint2(p[4], p[5]);
    pack_fp6(k2, p, mv.e2m1);
    uint32_t* d2 = op_q2 + (m * KB + b) * 8;
    reinterpret_cast<uint4*>(d2)[0] = make_uint4(p[0], p[1], p[2], p[3]);
    reinterpret_cast<uint2*>(d2)[2] = make_uint2(p[4], p[5]);
    op_e8m0[m * KB + b] = ebyte;
  }
}

int launch_decompose_mxfp4(const uint16_t* x, int64_t M, int64_t K, int64_t ldx, uint8_t* abi_q1,
                           uint8_t* abi_q2, uint8_t* abi_e8m0, uint32_t* op_q1, uint32_t* op_q2,
                           uint8_t* op_e8m0, MxVariant mv, hipStream_t stream) {
  if (M == 0 || K == 0) return MSD_OK;
  const int KB = (int)(K / 32);
  const int aligned = ((reinterpret_cast<uintptr_t>(x) & 15) == 0 && (ldx % 8) == 0) ? 1 : 0;
  const int64_t total = M * KB;
  hipLaunchKernelGGL(decompose_mxfp4_kernel, dim3((unsigned)cdiv(total, 256)), dim3(256), 0, stream,
                     x, ldx, M, KB, abi_q1, abi_q2, abi_e8m0, op_q1, op_q2, op_e8m0, aligned, mv);
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

}  // namespace msd
