// Comparison kernel for attention decode over an INT8 KV cache: the conventional path the paper
// argues against (Sec. 4.1: K and V are lifted to BF16 before Q K^T and P V; Sec. 4.4 prices it
// per token), written as the fused GPU form so that the two paths differ only in what the paper
// changes.  Same flash-decode split, same tile loads, same online softmax and the same merge of
// the split partials as the MSD kernel; but every K and V byte is converted to BF16 on the vector
// ALU (exact: |v| <= 127 fits BF16's 8-bit significand), the products run on
// v_mfma_f32_16x16x32_bf16, and P is rounded to BF16 (8 bits) instead of being split into two INT8
// components (16 bits).  The scales are applied where a careful dequantising kernel would apply
// them: per-token s_K[t] on the score column and s_V[t] on P in fp32 (equal to scaling the
// dequantised rows, without rounding them), per-channel s_K folded into Q (rounded to BF16) and
// s_V on the output.
//
// Fragment layouts (16 x 16 x 32: A lane = row l%16, 8 contraction slots of group l/16; D lane =
// column l%16, rows 4*(l/16) + r).  The contraction order is free as long as both operands agree:
//   Q K^T: slot i of group g in step (s, h) is channel 64 s + 16 g + 8 h + i, so a lane's 16 K
//          bytes (one 16-byte load) feed two steps;
//   P V:   slot 4 t2 + jq of group g in step u is token 16 (2u + t2) + 4 g + jq of the tile, which
//          is how the V loads of the MSD kernel already distribute the tokens over the lanes.
#include "attn_common.hpp"

namespace msd {

namespace {

union Bf8 {
  uint32_t u[4];
  v8bf v;
};

typedef float v2f_t __attribute__((ext_vector_type(2)));
typedef __bf16 v2bf_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi) {  // RNE, hardware convert
  const v2f_t f = {lo, hi};
  const v2bf_t b = __builtin_convertvector(f, v2bf_t);
  return *reinterpret_cast<const uint32_t*>(&b);
}
__device__ __forceinline__ float byte_f32(uint32_t w, int i) {  // signed byte i of w as float
  return (float)(int)(int8_t)((w >> (8 * i)) & 0xFFu);
}
__device__ __forceinline__ v4f mfma_bf(v8bf a, v8bf b, v4f c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

constexpr int kCmpHeads = 16;  // query heads per pass over the KV range: the 16 rows of the A fragment
constexpr int kPStride = 72;  // BF16 elements per head row of the P tile in LDS (64 + pad)

// MULTI (G > 16): the group is processed 16 heads at a time, one walk over the KV range each.
template <bool PER_TOKEN, bool MULTI>
__global__ __launch_bounds__(kAttnWaves * 64) void attn_dequant_kernel(AttnParams p) {
  __shared__ __attribute__((aligned(16))) uint16_t sQ[16][kD];
  __shared__ __attribute__((aligned(16))) uint16_t sP[kAttnWaves][16][kPStride];
  __shared__ float sM[kAttnWaves][kCmpHeads], sL[kAttnWaves][kCmpHeads];
  __shared__ float sO[kAttnWaves][kCmpHeads][kD];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 15, g = lane >> 4;
  const int bk = blockIdx.x / p.nsplit, split = blockIdx.x % p.nsplit;
  const int b = bk / p.Hkv, hk = bk % p.Hkv;
  const int G = p.G;
  int64_t len = p.kv_len ? (int64_t)p.kv_len[b] : p.L;
  len = max((int64_t)0, min(len, p.L));
  const int64_t t_begin = (int64_t)split * p.tokens_per_split;
  const int64_t t_end = min(len, t_begin + p.tokens_per_split);
  const int64_t kv_base = (int64_t)bk * p.L;
  const int8_t* Kb = p.K + kv_base * kD;
  const int8_t* Vb = p.V + kv_base * kD;

  const float sm_scale = kLog2e / sqrtf((float)kD);  // scores are kept in log2 units
  const v4f zero4f = {0.f, 0.f, 0.f, 0.f};
  const int64_t last = max(t_end - 1, (int64_t)0);
  const int64_t t_first = t_begin + (int64_t)wave * kTile;
  for (int h0 = 0; h0 < (MULTI ? G : 1); h0 += kCmpHeads) {  // one pass over the KV range per 16 heads
  // ---- prologue: the query rows as BF16 (per-channel mode: Q * s_K rounded to BF16), zero rows above G
  for (int idx = tid; idx < 16 * kD; idx += kAttnWaves * 64) {
    const int h = idx / kD, c = idx % kD;
    uint16_t v = 0;
    if (h0 + h < G) {
      v = p.q[((int64_t)b * p.Hq + hk * G + h0 + h) * kD + c];
      if (!PER_TOKEN) v = f32_to_bf16_bits(__uint_as_float((uint32_t)v << 16) * p.k_scale[hk * kD + c]);
    }
    sQ[h][c] = v;
  }
  __syncthreads();
  Bf8 qa[2][2];
#pragma unroll
  for (int s = 0; s < 2; ++s)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint4 v = *reinterpret_cast<const uint4*>(&sQ[j][64 * s + 16 * g + 8 * h]);
      qa[s][h].u[0] = v.x; qa[s][h].u[1] = v.y; qa[s][h].u[2] = v.z; qa[s][h].u[3] = v.w;
    }

  // per-lane state as a D lane: heads h0 + 4 g + r, r = 0..3
  float m_run[4], l_run[4], o_run[8][4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    m_run[r] = -INFINITY;
    l_run[r] = 0.f;
#pragma unroll
    for (int c = 0; c < 8; ++c) o_run[c][r] = 0.f;
  }
  // tile loads, software-pipelined exactly as in the MSD kernel
  v4i kf[4][2], kfn[4][2];
  v2i vr[4][4], vrn[4][4];  // [jq][tt]: 8 channels (8j..8j+7) of token 16*tt + 4*g + jq
  float sk[4], sv[4], skn[4], svn[4];
  auto load_tile = [&](int64_t t0, v4i (&kx)[4][2], v2i (&vx)[4][4], float (&skx)[4], float (&svx)[4]) {
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) {
      const int64_t tok = min(t0 + 16 * tt + j, last);
#pragma unroll
      for (int s = 0; s < 2; ++s)
        kx[tt][s] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(Kb + tok * kD + 64 * s + 16 * g));
    }
#pragma unroll
    for (int jq = 0; jq < 4; ++jq)
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) {
        const int64_t tok = min(t0 + 16 * tt + 4 * g + jq, last);
        vx[jq][tt] = __builtin_nontemporal_load(reinterpret_cast<const v2i*>(Vb + tok * kD + 8 * j));
      }
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) {
      skx[tt] = 1.f;
      svx[tt] = 1.f;
      if (PER_TOKEN) {
        const int64_t tok = min(t0 + 16 * tt + j, last);
        skx[tt] = p.k_scale[kv_base + tok];
        svx[tt] = p.v_scale[kv_base + tok];
      }
    }
  };
  if (t_first < t_end) load_tile(t_first, kfn, vrn, skn, svn);
  for (int64_t t0 = t_first; t0 < t_end; t0 += kAttnWaves * kTile) {
    bool live[4];
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) {
      live[tt] = t0 + 16 * tt + j < t_end;
      sk[tt] = skn[tt];
      sv[tt] = live[tt] ? svn[tt] : 0.f;
#pragma unroll
      for (int s = 0; s < 2; ++s) kf[tt][s] = kfn[tt][s];
#pragma unroll
      for (int jq = 0; jq < 4; ++jq) vr[jq][tt] = vrn[jq][tt];
    }
    if (t0 + kAttnWaves * kTile < t_end) load_tile(t0 + kAttnWaves * kTile, kfn, vrn, skn, svn);
    // ---- K tile to BF16, S = Q K^T
    v4f sd[4];
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) {
      sd[tt] = zero4f;
#pragma unroll
      for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          Bf8 kb;
#pragma unroll
          for (int d = 0; d < 2; ++d) {
            const uint32_t w = (uint32_t)kf[tt][s][2 * h + d];
            kb.u[2 * d] = pack2_bf16(byte_f32(w, 0), byte_f32(w, 1));
            kb.u[2 * d + 1] = pack2_bf16(byte_f32(w, 2), byte_f32(w, 3));
          }
          sd[tt] = mfma_bf(qa[s][h].v, kb.v, sd[tt]);
        }
    }
    // ---- online softmax; P (times s_V) to BF16
    float corr[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float sc[4];
      float mx = -INFINITY;
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) {
        const float v = sd[tt][r] * (sm_scale * sk[tt]);
        sc[tt] = live[tt] ? v : -INFINITY;
        mx = fmaxf(mx, sc[tt]);
      }
      mx = row16_max(mx);
      const float m_new = fmaxf(m_run[r], mx);
      corr[r] = __builtin_amdgcn_exp2f(m_run[r] - m_new);
      m_run[r] = m_new;
      float lsum = 0.f;
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) {
        const float pr = __builtin_amdgcn_exp2f(sc[tt] - m_new);
        lsum += pr;
        sP[wave][4 * g + r][16 * tt + j] = f32_to_bf16_bits(pr * sv[tt]);
      }
      l_run[r] = l_run[r] * corr[r] + lsum;
    }
    __builtin_amdgcn_wave_barrier();
    Bf8 pa[2];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        const uint2 v = *reinterpret_cast<const uint2*>(&sP[wave][j][16 * (2 * u + t2) + 4 * g]);
        pa[u].u[2 * t2] = v.x;
        pa[u].u[2 * t2 + 1] = v.y;
      }
    __builtin_amdgcn_wave_barrier();
    // ---- V tile to BF16 (channel 8j + c of the 16 tokens this lane holds), O += P V
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      v4f od = zero4f;
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        Bf8 vb;
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
          const int tt = 2 * u + t2;
          float f[4];
#pragma unroll
          for (int jq = 0; jq < 4; ++jq) f[jq] = byte_f32((uint32_t)vr[jq][tt][c >> 2], c & 3);
          vb.u[2 * t2] = pack2_bf16(f[0], f[1]);
          vb.u[2 * t2 + 1] = pack2_bf16(f[2], f[3]);
        }
        od = mfma_bf(pa[u].v, vb.v, od);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) o_run[c][r] = o_run[c][r] * corr[r] + od[r];
    }
  }

  // ---- merge the waves of this workgroup, write the split's partial (m, l, O)
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const float lt = row16_sum(l_run[r]);
    const int hs = 4 * g + r;
    if (j == 0) {
      sM[wave][hs] = m_run[r];
      sL[wave][hs] = lt;
    }
#pragma unroll
    for (int c = 0; c < 8; ++c) sO[wave][hs][8 * j + c] = o_run[c][r];
  }
  __syncthreads();
  const int nh_here = min(kCmpHeads, G - h0);
  for (int idx = tid; idx < nh_here * kD; idx += kAttnWaves * 64) {
    const int hl = idx / kD, c = idx % kD;
    const int h = h0 + hl;
    float ms = -INFINITY;
#pragma unroll
    for (int w = 0; w < kAttnWaves; ++w) ms = fmaxf(ms, sM[w][hl]);
    float o = 0.f, l = 0.f;
#pragma unroll
    for (int w = 0; w < kAttnWaves; ++w) {
      const float wgt = (sM[w][hl] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(sM[w][hl] - ms);
      o += sO[w][hl][c] * wgt;
      l += sL[w][hl] * wgt;
    }
    if (p.nsplit == 1) {
      float v = l > 0.f ? __fdiv_rn(o, l) : 0.f;
      if (!PER_TOKEN) v *= p.v_scale[hk * kD + c];
      const int64_t orow = (int64_t)b * p.Hq + hk * G + h;
      if (p.out_bf16)
        reinterpret_cast<uint16_t*>(p.out)[orow * kD + c] = f32_to_bf16_bits(v);
      else
        reinterpret_cast<float*>(p.out)[orow * kD + c] = v;
    } else {
      const int64_t pr = ((int64_t)bk * p.nsplit + split) * G + h;
      p.part_o[pr * kD + c] = o;
      if (c == 0) {
        p.part_m[pr] = ms;
        p.part_l[pr] = l;
      }
    }
  }
  if (MULTI && h0 + kCmpHeads < G) __syncthreads();  // sQ and the merge buffers are reused by the next head group
  }
}

}  // namespace

int launch_attn_dequant(const AttnArgs& a, hipStream_t stream) {
  AttnParams p{};
  attn_fill_params(a, p);
  const dim3 grid((unsigned)((int64_t)a.B * a.Hkv * p.nsplit));
  const bool per_token = a.scale_mode == MSD_PER_TOKEN;
  if (p.G <= kCmpHeads) {
    if (per_token)
      hipLaunchKernelGGL((attn_dequant_kernel<true, false>), grid, dim3(kAttnWaves * 64), 0, stream, p);
    else
      hipLaunchKernelGGL((attn_dequant_kernel<false, false>), grid, dim3(kAttnWaves * 64), 0, stream, p);
  } else {
    if (per_token)
      hipLaunchKernelGGL((attn_dequant_kernel<true, true>), grid, dim3(kAttnWaves * 64), 0, stream, p);
    else
      hipLaunchKernelGGL((attn_dequant_kernel<false, true>), grid, dim3(kAttnWaves * 64), 0, stream, p);
  }
  MSD_LAUNCH_CHECK();
  if (p.nsplit > 1) return launch_attn_combine(p, per_token ? 0 : 1, stream);
  return MSD_OK;
}

}  // namespace msd
