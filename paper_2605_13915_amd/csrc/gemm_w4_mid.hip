// W4A16 MSD GEMM for 32 activation rows or fewer when the weight stream is the bound (batched
// decode): paper Sec. 3.2.1 / Alg. 2 feeding Sec. 3.4.1 on v_mfma_scale_f32_32x32x64_f8f6f4.
//
// Two launches per call: the K-step-major decomposition of gemm_w4_prefill.hip (one group of 32
// rows: 3 KB of FP6 operands and 64 scale bytes per K step of 64 elements), then this kernel.
//
// One workgroup = 4 waves = 128 output channels, the whole K range, all rows; a wave owns 32
// channels (lane l: channel l%32, MX block l/32 of each K step).  K is walked in batches of U steps.
// Per batch the workgroup stages 32 KB of weights (128 channels x 256 B, fetched 256 contiguous
// bytes per channel and instruction) and the activation operands of the batch (U * 3 KB + scale
// bytes, hot in L2, shared by the four waves) through LDS, double-buffered: global -> registers at
// the start of a batch, registers -> LDS after its MFMAs, one barrier per batch.  Weight rows sit in
// LDS with a 16-byte pad per 256 bytes, which makes both the staging stores (16 lanes per row) and
// the fragment reads (32 rows at one K offset) conflict-free.  The weights' scale bytes (16 per
// channel and batch) go straight to registers.  Both components accumulate into one fp32
// accumulator of 16 registers (scale bytes alpha and alpha - shift).
// Why not weights straight into the B operand, as in the skinny kernel: with the 32 x 32 x 64
// instruction only two lanes share a weight row, so every load instruction touches 32 rows with 32
// bytes each -- measured 55 us (cacheable) to 68 us (non-temporal) at M = 32, N = 28672, K = 8192,
// against the skinny kernel's re-reading of the activation operands per 16 channels at 78 us.
#include "kernels.hpp"

namespace msd {

namespace {

constexpr int kMidU = 8;  // K steps per batch (256 weight bytes per channel)
constexpr int kMidThreads = 256;
constexpr int kMidBN = 128;                                   // channels per workgroup
constexpr int kMidStageA = kMidU * 3072 / 16 / kMidThreads;   // 16-byte activation-operand chunks per thread and batch
constexpr int kMidStageW = kMidBN * kMidU * 32 / 16 / kMidThreads;  // 16-byte weight chunks per thread and batch
constexpr int kMidRowW = kMidU * 32 + 16;                     // LDS bytes per weight row (padded)
constexpr int kMidBufA = kMidU * (3072 + 256);                // operands, then the scale dwords
constexpr int kMidBufW = kMidBN * kMidRowW;
constexpr int kMidLds = 2 * (kMidBufA + kMidBufW);
static_assert(kMidStageA * kMidThreads * 16 == kMidU * 3072 && kMidU * 16 <= kMidThreads, "batch split");
static_assert(kMidU * 32 / 16 == 16, "a weight row of a batch is 16 chunks: 16 lanes per row");

__device__ __forceinline__ v16f mfma_mid(v8i a, v8i b, v16f c, int sa, int sb) {
  // A: FP6 E2M3 (cbsz = 2), B: FP4 E2M1 (blgp = 4); E8M0 scales in byte 0 of sa / sb
  return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 2, 4, 0, sa, 0, sb);
}

__global__ __launch_bounds__(kMidThreads) void gemm_w4_mid_kernel(const uint8_t* __restrict__ qop,
                                                                  const uint8_t* __restrict__ sa_t,
                                                                  const uint8_t* __restrict__ W,
                                                                  const uint8_t* __restrict__ We, void* y,
                                                                  int out_bf16, int64_t ldy, int M, int64_t K,
                                                                  int64_t N, int shift) {
  extern __shared__ __attribute__((aligned(16))) uint8_t s_mid[];  // [2][A batch] then [2][W batch]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, kb = lane >> 5;
  const int64_t n0 = (int64_t)blockIdx.x * kMidBN;
  const int64_t n = n0 + wave * 32 + l32;
  // channels past N repeat the last one; their results are not stored
  const uint8_t* werow = We + min(n, N - 1) * (K / 32);
  const int NB = (int)(K / (64 * kMidU));  // batches (K is a multiple of 64 * kMidU)
  // weight staging: chunk tid + i * 256 of the batch = (row r = chunk / 16, 16-byte column c = chunk % 16)
  const int wr = tid >> 4, wc = tid & 15;
  const uint8_t* wsrc[kMidStageW];
#pragma unroll
  for (int i = 0; i < kMidStageW; ++i) wsrc[i] = W + min(n0 + wr + 16 * i, N - 1) * (K / 2) + wc * 16;

  // two register stages: while batch b is multiplied out of LDS, batch b + 1 and batch b + 2 are in flight
  struct Stage {
    v4i w[kMidStageW], a[kMidStageA], asc, wsc;  // wsc: the 16 weight scale bytes of this lane's channel
  };
  Stage st0, st1;
  st0.asc = st1.asc = v4i{0, 0, 0, 0};
  auto load_batch = [&](int b, Stage& st) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < kMidStageW; ++i)
      st.w[i] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(wsrc[i] + (int64_t)b * (kMidU * 32)));
    st.wsc = *reinterpret_cast<const v4i*>(werow + (int64_t)b * 16);
    const uint8_t* src = qop + (int64_t)b * (kMidU * 3072);  // the batch's operands are contiguous
#pragma unroll
    for (int i = 0; i < kMidStageA; ++i) st.a[i] = *reinterpret_cast<const v4i*>(src + (tid + i * kMidThreads) * 16);
    // scale dwords: 256 of each step's 512-byte record, one 16-byte chunk per thread of the first two waves
    if (tid < kMidU * 16)
      st.asc = *reinterpret_cast<const v4i*>(sa_t + ((int64_t)b * kMidU + (tid >> 4)) * 512 + (tid & 15) * 16);
  };
  auto store_batch = [&](int buf, const Stage& st) __attribute__((always_inline)) {
    uint8_t* sa = s_mid + buf * kMidBufA;
    uint8_t* sw = s_mid + 2 * kMidBufA + buf * kMidBufW;
#pragma unroll
    for (int i = 0; i < kMidStageW; ++i) *reinterpret_cast<v4i*>(sw + (wr + 16 * i) * kMidRowW + wc * 16) = st.w[i];
#pragma unroll
    for (int i = 0; i < kMidStageA; ++i) *reinterpret_cast<v4i*>(sa + (tid + i * kMidThreads) * 16) = st.a[i];
    if (tid < kMidU * 16) *reinterpret_cast<v4i*>(sa + kMidU * 3072 + tid * 16) = st.asc;
  };
  v16f acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  auto multiply = [&](int buf, const v4i& sc) __attribute__((always_inline)) {
    const uint8_t* sa_buf = s_mid + buf * kMidBufA;
    const uint8_t* sw_row = s_mid + 2 * kMidBufA + buf * kMidBufW + (wave * 32 + l32) * kMidRowW + kb * 16;
#pragma unroll
    for (int u = 0; u < kMidU; ++u) {
      const uint8_t* rec = sa_buf + u * 3072;
      const int sa = *reinterpret_cast<const int*>(sa_buf + kMidU * 3072 + u * 256 + kb * 128 + l32 * 4) & 0xFF;
      // scale byte of block 2u + kb of the batch
      const uint32_t sw = (uint32_t)(u < 2 ? sc[0] : u < 4 ? sc[1] : u < 6 ? sc[2] : sc[3]);
      const int sb = (int)((sw >> (16 * (u & 1) + 8 * kb)) & 0xFFu);
      const v4i w = *reinterpret_cast<const v4i*>(sw_row + u * 32);
      const v8i bw = {w[0], w[1], w[2], w[3], 0, 0, 0, 0};
#pragma unroll
      for (int comp = 0; comp < 2; ++comp) {
        const uint4 lo = *reinterpret_cast<const uint4*>(rec + ((3 * comp + kb) * 32 + l32) * 16);
        const uint2 hi = *reinterpret_cast<const uint2*>(rec + ((3 * comp + 2) * 32 + l32) * 16 + kb * 8);
        const v8i av = {(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, 0, 0};
        acc = mfma_mid(av, bw, acc, sa - shift * comp, sb);  // beta = alpha / 2^shift
      }
    }
  };

  // LDS buffer b % 2 and register stage b % 2 belong to batch b; the scale bytes of a batch stay in
  // its register stage until the batch after next is fetched into it, i.e. until it has been multiplied
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

}  // namespace

bool gemm_w4_mid_applies(int64_t M, int64_t K, int64_t N, bool scales_aligned) {
  // whole batches of K steps; 16-byte loads of the weight scale rows
  return M > 4 && M <= 32 && N >= 1 && K >= 64 * kMidU && K % (64 * kMidU) == 0 && scales_aligned;
}

W4MidLayout w4_mid_layout(int64_t K) {
  W4MidLayout l{};
  const size_t steps = (size_t)K / 64;
  size_t off = 0;
  l.qop = off; off = align_up(off + steps * 3072, 256);
  l.sa_t = off; off = align_up(off + steps * 512, 256);
  l.total = off;
  return l;
}

int launch_gemm_w4_mid(const uint16_t* x, int64_t ldx, const uint8_t* W, const uint8_t* We, void* y, int out_bf16,
                       int64_t ldy, int64_t M, int64_t K, int64_t N, uint8_t* ws, MxVariant mv, hipStream_t stream) {
  const W4MidLayout l = w4_mid_layout(K);
  if (int rc = launch_decompose_mxfp4_pair(x, ldx, M, K, 32, ws + l.qop, ws + l.sa_t, mv, stream)) return rc;
  static bool attr_set = false;
  if (!attr_set) {
    MSD_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_w4_mid_kernel),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, kMidLds));
    attr_set = true;
  }
  hipLaunchKernelGGL(gemm_w4_mid_kernel, dim3((unsigned)cdiv(N, kMidBN)), dim3(kMidThreads), kMidLds, stream,
                     ws + l.qop, ws + l.sa_t, W, We, y, out_bf16, ldy, (int)M, K, N, mv.shift);
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

}  // namespace msd
