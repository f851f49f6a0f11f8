// Measurement aid, not part of the method: a bare read of a row-major byte matrix in the access
// pattern of the decode kernels' weight stream (a workgroup owns 16 rows, its four waves split
// the row, each wave instruction fetches 16 rows x 64 B, eight instructions in flight per lane).
// Nothing is computed or written.  Its time is what the same bytes cost on this GPU with no
// arithmetic at all, launch included: the floor the decode kernels are measured against.
#include "kernels.hpp"

namespace msd {

__device__ int g_stream_probe_sink;

__global__ __launch_bounds__(256) void stream_read_kernel(const int8_t* __restrict__ src, int64_t rows,
                                                          int64_t row_bytes) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row = min((int64_t)blockIdx.x * 16 + (lane & 15), rows - 1);
  const int64_t quarter = row_bytes / 4;  // row_bytes % 256 == 0 (checked on the host)
  const int8_t* p = src + row * row_bytes + wave * quarter + 16 * (lane >> 4);
  v4i acc = {0, 0, 0, 0};
  for (int64_t k0 = 0; k0 < quarter; k0 += 64 * 8) {
    v4i r[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int64_t k = min(k0 + 64 * u, quarter - 64);  // the tail re-reads the last 64-byte column
      r[u] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(p + k));
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= r[u];
  }
  // keeps the loads alive; the condition is practically never true and the value is never read
  if (acc[0] == 0x5EEDBEEF && acc[1] == 0x0BADF00D && acc[2] == acc[3]) g_stream_probe_sink = acc[2];
}

// The same bytes as one linear array: a wave instruction fetches one contiguous kilobyte (the pattern of the
// packed weight layouts), sixteen instructions in flight per lane, 64 KB per workgroup.
__global__ __launch_bounds__(256) void stream_read_linear_kernel(const int8_t* __restrict__ src, int64_t bytes) {
  const int64_t base = (int64_t)blockIdx.x * 65536 + threadIdx.x * 16;
  v4i acc = {0, 0, 0, 0};
  v4i r[16];
#pragma unroll
  for (int u = 0; u < 16; ++u) {
    const int64_t off = min(base + u * 4096, bytes - 16);  // the tail re-reads the last 16 bytes
    r[u] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(src + off));
  }
#pragma unroll
  for (int u = 0; u < 16; ++u) acc ^= r[u];
  if (acc[0] == 0x5EEDBEEF && acc[1] == 0x0BADF00D && acc[2] == acc[3]) g_stream_probe_sink = acc[2];
}

int launch_stream_read_linear(const void* src, int64_t bytes, hipStream_t stream) {
  if (bytes == 0) return MSD_OK;
  hipLaunchKernelGGL(stream_read_linear_kernel, dim3((unsigned)cdiv(bytes, 65536)), dim3(256), 0, stream,
                     (const int8_t*)src, bytes);
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

// ------------------------------------------------------------------ matrix-pipe rate
// Nothing but matrix instructions: every wave loads four A and two B operand fragments (16 bytes per lane each; 24
// bytes for the FP6 A fragments) from `operands` once and then issues `iters` rounds of the eight products
// A_i x B_j into eight independent accumulators -- the instruction pattern of the many-row GEMM kernels with no
// data movement at all.  What it measures is how fast the matrix pipe runs ON THESE OPERAND BITS: the
// instruction rate in cycles is fixed, the clock the chip sustains under the load is not.
typedef int v16i_probe __attribute__((ext_vector_type(16)));
typedef float v16f_probe __attribute__((ext_vector_type(16)));
template <bool FP4>
__global__ __launch_bounds__(128) void mfma_rate_kernel(const int* __restrict__ operands, int iters) {
  const v4i* src = reinterpret_cast<const v4i*>(operands);
  v4i A[4], A2[4], B[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    A[i] = src[(threadIdx.x * 10 + i) & 4095];
    A2[i] = src[(threadIdx.x * 10 + 6 + i) & 4095];
  }
#pragma unroll
  for (int j = 0; j < 2; ++j) B[j] = src[(threadIdx.x * 10 + 4 + j) & 4095];
  int sink = 0;
  if constexpr (FP4) {
    v16f_probe acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const v8i a8 = {A[i][0], A[i][1], A[i][2], A[i][3], A2[i][0], A2[i][1], 0, 0};
          const v8i b8 = {B[j][0], B[j][1], B[j][2], B[j][3], 0, 0, 0, 0};
          // FP6 x FP4, scale bytes 2^0 (every bit pattern of both element formats is a finite number)
          acc[i * 2 + j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, acc[i * 2 + j], 2, 4, 0, 0x7F7F7F7F, 0, 0x7F7F7F7F);
        }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) sink += (int)acc[i][0];
  } else {
    v16i_probe acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i * 2 + j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[i], B[j], acc[i * 2 + j], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) sink += acc[i][0];
  }
  if (sink == 0x5EEDBEEF && iters < 0) g_stream_probe_sink = sink;  // keeps the products alive; never true
}

int launch_mfma_rate(int fp4, const void* operands, int iters, hipStream_t stream) {
  const dim3 grid(1024), block(128);  // eight waves per CU, two per SIMD
  if (fp4)
    hipLaunchKernelGGL(mfma_rate_kernel<true>, grid, block, 0, stream, (const int*)operands, iters);
  else
    hipLaunchKernelGGL(mfma_rate_kernel<false>, grid, block, 0, stream, (const int*)operands, iters);
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

// ------------------------------------------------------------------ LDS fill rate
// Nothing but the fill instructions of the tile kernels: one workgroup of eight waves per CU; per round a wave
// issues four asynchronous 16-byte-per-lane loads into LDS (one contiguous kilobyte each, 32 KB per workgroup and
// round) into a ring of four rounds, and before it issues round r + 2 it waits for its loads of round r and meets
// the other waves at a barrier -- the issue pattern, depth and synchronisation of gemm_w8_dma_kernel with no
// fragment reads and no matrix instructions.  Of the four instructions the first `hot_parts` read a window at the
// start of `src` that every workgroup walks in the same order (the activation codes, which come from L2); the
// others read the rest of `src`, every workgroup its own range (the weight stream, which comes from HBM).  Its
// time is what moving those bytes into LDS costs with no arithmetic at all.
__device__ __forceinline__ void probe_lds_dma16(const int8_t* gbase, uint32_t voff, uint32_t lds_addr) {
  const uint64_t g = reinterpret_cast<uint64_t>(gbase);
  const uint32_t glo = __builtin_amdgcn_readfirstlane((uint32_t)g), ghi = __builtin_amdgcn_readfirstlane((uint32_t)(g >> 32));
  gbase = reinterpret_cast<const int8_t*>(((uint64_t)ghi << 32) | glo);
  lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(voff), "s"(gbase), "s"(lds_addr)
               : "memory", "m0");
}

constexpr int kFillProbeRing = 4, kFillProbeRound = 32768;

__global__ __launch_bounds__(512) void lds_fill_rate_kernel(const int8_t* __restrict__ src, int64_t hot_kb, int64_t cold_kb,
                                                            int hot_parts, int rounds) {
  extern __shared__ __attribute__((aligned(16))) int8_t fill_ring[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
  const uint32_t lds0 = (uint32_t)(uintptr_t)fill_ring;
  const uint32_t voff = (uint32_t)(lane * 16);
  auto issue = [&](int r) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int i = q * 8 + wave;  // kilobyte of the round
      int64_t kb;
      if (q < hot_parts) kb = ((int64_t)r * 32 + i) % hot_kb;
      else kb = hot_kb + (((int64_t)blockIdx.x * rounds + r) * 32 + i) % cold_kb;
      probe_lds_dma16(src + kb * 1024, voff, lds0 + (uint32_t)((r % kFillProbeRing) * kFillProbeRound + i * 1024));
    }
  };
  if (rounds > 0) issue(0);
  if (rounds > 1) issue(1);
  for (int r = 0; r < rounds; ++r) {
    // loads of rounds r + 1 (and nothing younger) may stay outstanding; at the end everything drains
    if (r + 1 < rounds) asm volatile("s_waitcnt vmcnt(4)\n\ts_barrier" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    if (r + 2 < rounds) issue(r + 2);
  }
  // one LDS word per workgroup is read back so that the fills cannot be dropped; the condition is never true
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (threadIdx.x == 0 && rounds < 0) g_stream_probe_sink = reinterpret_cast<const int*>(fill_ring)[lane];
}

int launch_lds_fill_rate(const void* src, int64_t src_bytes, int64_t hot_bytes, int hot_parts, int rounds,
                         hipStream_t stream) {
  constexpr int kLds = kFillProbeRing * kFillProbeRound;
  static bool attr_set = false;
  if (!attr_set) {
    MSD_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&lds_fill_rate_kernel),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, kLds));
    attr_set = true;
  }
  hipLaunchKernelGGL(lds_fill_rate_kernel, dim3(256), dim3(512), kLds, stream, (const int8_t*)src, hot_bytes / 1024,
                     (src_bytes - hot_bytes) / 1024, hot_parts, rounds);
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

int launch_stream_read(const void* src, int64_t rows, int64_t row_bytes, hipStream_t stream) {
  if (rows == 0 || row_bytes == 0) return MSD_OK;
  hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)cdiv(rows, 16)), dim3(256), 0, stream,
                     (const int8_t*)src, rows, row_bytes);
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

}  // namespace msd
