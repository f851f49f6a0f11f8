// MSD attention decode over an INT8 latent KV cache (multi-head latent attention; paper Sec. 4.2 /
// Alg. 3 with the shapes of Sec. 4.4 and Sec. 7.3: 512 latent channels plus 64 positional ones).
// One cached row per token serves every query head of a batch entry: its 576 channels are the key,
// its first 512 the value.  The steps are those of the grouped-query kernel (attn.hip) -- Q rows
// decomposed once, S1 / S2 on v_mfma_i32_16x16x64_i8 with [Q1; Q2] stacked, merge, online softmax in
// fp32, P decomposed with a scale that needs no reduction over P, O1 / O2 on the same instruction
// with V transposed in registers -- reshaped for the wide rows:
//   * the key product walks the 576 channels in nine 64-channel chunks, three chunks in flight;
//   * the value product walks the 512 channels in four 128-channel slabs; the running output of the
//     8 heads of a pass is 64 registers per lane;
//   * the cached rows are read twice per tile (as key chunks, then as value slabs, in the two
//     operand layouts); the second read hits L2, HBM sees each row once per pass;
//   * 8 query heads share a pass over the KV range (one 16-row A fragment: 8 heads x 2 components);
//     more heads are processed 8 at a time, re-decomposing their Q rows per pass.
// The KV length is split over workgroups; a second kernel merges the split partials.
#include "attn_common.hpp"

namespace msd {

namespace {

constexpr int kLatK = 576;  // key channels (latent + positional)
constexpr int kLatV = 512;  // value channels (latent)
constexpr int kLatHeads = 8;

struct MlaParams {
  const uint16_t* q;   // [B][Hq][576]
  const int8_t* C;     // [B][L][ld]
  const float* scale;  // per token [B][L] or per channel [576]
  const int32_t* kv_len;
  int B, Hq;
  int64_t L, ld;
  int nsplit;
  int64_t tokens_per_split;
  float sm_scale_log2;  // score scale times log2(e)
  float* part_o;        // [B][nsplit][Hq][512]
  float* part_m;        // [B][nsplit][Hq]
  float* part_l;
  void* out;
  int out_bf16;
  int8_t* tap_q1;
  int8_t* tap_q2;
  float* tap_alpha;
  int32_t* tap_s1;
  int32_t* tap_s2;
};

template <bool PER_TOKEN>
__global__ __launch_bounds__(kAttnWaves * 64) void attn_mla_kernel(MlaParams p) {
  constexpr int NH = kLatHeads;
  // LDS (dynamic): sO[waves][NH][512] f32 | sQ[2][NH][576] int8 | sP[waves][2][NH][16] u32 | sAlpha[NH] |
  // sM[waves][NH] | sL[waves][NH]
  extern __shared__ __attribute__((aligned(16))) uint8_t s_mla[];
  float(*sO)[NH][kLatV] = reinterpret_cast<float(*)[NH][kLatV]>(s_mla);
  int8_t(*sQ)[NH][kLatK] = reinterpret_cast<int8_t(*)[NH][kLatK]>(s_mla + kAttnWaves * NH * kLatV * 4);
  uint32_t(*sP)[2][NH][16] =
      reinterpret_cast<uint32_t(*)[2][NH][16]>(s_mla + kAttnWaves * NH * kLatV * 4 + 2 * NH * kLatK);
  float* sAlpha = reinterpret_cast<float*>(s_mla + kAttnWaves * NH * kLatV * 4 + 2 * NH * kLatK +
                                           kAttnWaves * 2 * NH * 64);
  float(*sM)[NH] = reinterpret_cast<float(*)[NH]>(sAlpha + NH);
  float(*sL)[NH] = sM + kAttnWaves;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 15, g = lane >> 4;
  const int b = blockIdx.x / p.nsplit, split = blockIdx.x % p.nsplit;
  const int Hq = p.Hq;
  int64_t len = p.kv_len ? (int64_t)p.kv_len[b] : p.L;
  len = max((int64_t)0, min(len, p.L));
  const int64_t t_begin = (int64_t)split * p.tokens_per_split;
  const int64_t t_end = min(len, t_begin + p.tokens_per_split);
  const int64_t last = max(t_end - 1, (int64_t)0);
  const int8_t* Cb = p.C + (int64_t)b * p.L * p.ld;
  const float* sc_tok = p.scale + (int64_t)b * p.L;  // per-token mode only
  const int64_t t_first = t_begin + (int64_t)wave * kTile;
  const v4i zero4 = {0, 0, 0, 0};

  // A-fragment row of this lane: slot j&3 of head pair j>>2 = (head, component)
  const int slot = j & 3;
  const int row_head = (j >> 2) * 2 + (slot >> 1);
  const int row_comp = slot & 1;

  for (int h0 = 0; h0 < Hq; h0 += NH) {  // one pass over the KV range per 8 heads
    // ---- decompose the query rows of this pass (Alg. 3 steps 1-2), two heads per wave
    for (int h = wave; h < NH; h += kAttnWaves) {
      float x[9];
      float mx = 0.f;
      const bool live_head = h0 + h < Hq;
      const int64_t qrow = (int64_t)b * Hq + h0 + h;
#pragma unroll
      for (int i = 0; i < 9; ++i) {
        const int c = lane + 64 * i;
        x[i] = 0.f;
        if (live_head) {
          x[i] = __uint_as_float((uint32_t)p.q[qrow * kLatK + c] << 16);
          if (!PER_TOKEN) x[i] *= p.scale[c];  // absorb the per-channel key scale into Q
        }
        mx = fmaxf(mx, fabsf(x[i]));
      }
      mx = wave_max(mx);
      const float alpha = mx > 0.f ? __fdiv_rn(mx, 127.0f) : 0.f;
      const float beta = __fdiv_rn(alpha, 254.0f);
#pragma unroll
      for (int i = 0; i < 9; ++i) {
        const int c = lane + 64 * i;
        int c1 = 0, c2 = 0;
        if (mx > 0.f) int8_codes(x[i], alpha, beta, c1, c2);
        sQ[0][h][c] = (int8_t)c1;
        sQ[1][h][c] = (int8_t)c2;
        if (live_head && split == 0 && p.tap_q1) {
          p.tap_q1[qrow * kLatK + c] = (int8_t)c1;
          p.tap_q2[qrow * kLatK + c] = (int8_t)c2;
        }
      }
      if (lane == 0) {
        sAlpha[h] = alpha;
        if (live_head && split == 0 && p.tap_q1) p.tap_alpha[qrow] = alpha;
      }
    }
    __syncthreads();
    v4i qa[9];
#pragma unroll
    for (int s = 0; s < 9; ++s) qa[s] = *reinterpret_cast<const v4i*>(&sQ[row_comp][row_head][64 * s + 16 * g]);
    float aq[2], bq[2], m_run[2], l_run[2], o_run[4][2][8];
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      aq[hh] = sAlpha[g * 2 + hh];
      bq[hh] = __fdiv_rn(aq[hh], 254.0f);
      m_run[hh] = -INFINITY;
      l_run[hh] = 0.f;
#pragma unroll
      for (int sl = 0; sl < 4; ++sl)
#pragma unroll
        for (int c = 0; c < 8; ++c) o_run[sl][hh][c] = 0.f;
    }

    for (int64_t t0 = t_first; t0 < t_end; t0 += kAttnWaves * kTile) {
      bool live[4];
      int64_t tokK[4];
      float sk[4];
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) {
        live[tt] = t0 + 16 * tt + j < t_end;
        tokK[tt] = min(t0 + 16 * tt + j, last);
        sk[tt] = PER_TOKEN ? sc_tok[tokK[tt]] : 1.f;
      }
      // ---- (2) S1, S2: nine 64-channel chunks, three at a time
      v4i sd[4] = {zero4, zero4, zero4, zero4};
#pragma unroll
      for (int s3 = 0; s3 < 3; ++s3) {
        v4i kx[3][4];
#pragma unroll
        for (int u = 0; u < 3; ++u)
#pragma unroll
          for (int tt = 0; tt < 4; ++tt)
            kx[u][tt] = __builtin_nontemporal_load(
                reinterpret_cast<const v4i*>(Cb + tokK[tt] * p.ld + 64 * (3 * s3 + u) + 16 * g));
#pragma unroll
        for (int u = 0; u < 3; ++u)
#pragma unroll
          for (int tt = 0; tt < 4; ++tt) sd[tt] = mfma_s8(qa[3 * s3 + u], kx[u][tt], sd[tt]);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (p.tap_s1) {
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
          const int head = h0 + g * 2 + hh;
          if (head < Hq) {
            const int64_t row = ((int64_t)b * Hq + head) * p.L;
#pragma unroll
            for (int tt = 0; tt < 4; ++tt)
              if (live[tt]) {
                p.tap_s1[row + t0 + 16 * tt + j] = sd[tt][2 * hh];
                p.tap_s2[row + t0 + 16 * tt + j] = sd[tt][2 * hh + 1];
              }
          }
        }
      }
      // scale of the P decomposition: alpha_P = top/127, top a bound on P (times the value scale)
      float sv[4];
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) sv[tt] = live[tt] ? sk[tt] : 0.f;
      float top = 1.f;
      if (PER_TOKEN) top = row16_max(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])));
      const float to_code = top > 0.f ? __fdiv_rn(127.0f, top) : 0.f;
      const float from_code = top * (1.0f / 127.0f);
      // ---- (3)+(4) merge, online softmax, decompose P
      float corr[2];
      uint32_t pk1[2], pk2[2];
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        float s[4];
        float mx = -INFINITY;
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
          const float v = (aq[hh] * (float)sd[tt][2 * hh] + bq[hh] * (float)sd[tt][2 * hh + 1]) * (p.sm_scale_log2 * sk[tt]);
          s[tt] = live[tt] ? v : -INFINITY;
          mx = fmaxf(mx, s[tt]);
        }
        mx = row16_max(mx);
        const float m_new = fmaxf(m_run[hh], mx);
        corr[hh] = __builtin_amdgcn_exp2f(m_run[hh] - m_new);
        m_run[hh] = m_new;
        float lsum = 0.f;
        uint32_t w1 = 0, w2 = 0;
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
          const float pr = __builtin_amdgcn_exp2f(s[tt] - m_new);
          lsum += pr;
          const float t = pr * sv[tt] * to_code;
          const float c1 = fminf(rintf(t), 127.f);
          const float c2 = fminf(fmaxf(rintf((t - c1) * 254.0f), -127.f), 127.f);
          w1 |= ((uint32_t)(int)c1 & 0xFFu) << (8 * tt);
          w2 |= ((uint32_t)(int)c2 & 0xFFu) << (8 * tt);
        }
        l_run[hh] = l_run[hh] * corr[hh] + lsum;
        pk1[hh] = w1;
        pk2[hh] = w2;
      }
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        sP[wave][0][g * 2 + hh][j] = pk1[hh];
        sP[wave][1][g * 2 + hh][j] = pk2[hh];
      }
      __builtin_amdgcn_wave_barrier();
      const v4i pa = *reinterpret_cast<const v4i*>(&sP[wave][row_comp][row_head][4 * g]);
      __builtin_amdgcn_wave_barrier();
      // ---- (5) O1, O2 over four 128-channel slabs of the same rows
      int64_t tokV[4][4];
#pragma unroll
      for (int jq = 0; jq < 4; ++jq)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) tokV[jq][tt] = min(t0 + 16 * tt + 4 * g + jq, last) * p.ld + 8 * j;
#pragma unroll
      for (int sl = 0; sl < 4; ++sl) {
        v2i vr[4][4];  // [jq][tt]: channels 128 sl + 8j .. +7 of token 16 tt + 4 g + jq
#pragma unroll
        for (int jq = 0; jq < 4; ++jq)
#pragma unroll
          for (int tt = 0; tt < 4; ++tt)
            vr[jq][tt] = *reinterpret_cast<const v2i*>(Cb + tokV[jq][tt] + 128 * sl);
        uint32_t vb[8][4];
#pragma unroll
        for (int jq = 0; jq < 4; ++jq) {
          uint32_t lo[4], hi[4];
          transpose4x4((uint32_t)vr[jq][0][0], (uint32_t)vr[jq][1][0], (uint32_t)vr[jq][2][0], (uint32_t)vr[jq][3][0], lo);
          transpose4x4((uint32_t)vr[jq][0][1], (uint32_t)vr[jq][1][1], (uint32_t)vr[jq][2][1], (uint32_t)vr[jq][3][1], hi);
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            vb[c][jq] = lo[c];
            vb[4 + c][jq] = hi[c];
          }
        }
#pragma unroll
        for (int c = 0; c < 8; ++c) {
          const v4i bf = {(int)vb[c][0], (int)vb[c][1], (int)vb[c][2], (int)vb[c][3]};
          const v4i od = mfma_s8(pa, bf, zero4);
#pragma unroll
          for (int hh = 0; hh < 2; ++hh) {
            const float ot = from_code * ((float)od[2 * hh] + (float)od[2 * hh + 1] * (1.0f / 254.0f));
            o_run[sl][hh][c] = o_run[sl][hh][c] * corr[hh] + ot;
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }

    // ---- merge the waves of this workgroup, write the split's partial (m, l, O) of these heads
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      const float lt = row16_sum(l_run[hh]);
      const int hs = g * 2 + hh;
      if (j == 0) {
        sM[wave][hs] = m_run[hh];
        sL[wave][hs] = lt;
      }
#pragma unroll
      for (int sl = 0; sl < 4; ++sl)
#pragma unroll
        for (int c = 0; c < 8; ++c) sO[wave][hs][128 * sl + 8 * j + c] = o_run[sl][hh][c];
    }
    __syncthreads();
    const int nh_here = min(NH, Hq - h0);
    for (int idx = tid; idx < nh_here * kLatV; idx += kAttnWaves * 64) {
      const int hl = idx / kLatV, c = idx % kLatV;
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
        if (!PER_TOKEN) v *= p.scale[c];
        const int64_t orow = (int64_t)b * Hq + h;
        if (p.out_bf16)
          reinterpret_cast<uint16_t*>(p.out)[orow * kLatV + c] = f32_to_bf16_bits(v);
        else
          reinterpret_cast<float*>(p.out)[orow * kLatV + c] = v;
      } else {
        const int64_t pr = ((int64_t)b * p.nsplit + split) * Hq + h;
        p.part_o[pr * kLatV + c] = o;
        if (c == 0) {
          p.part_m[pr] = ms;
          p.part_l[pr] = l;
        }
      }
    }
    __syncthreads();  // sQ and the merge buffers are rewritten by the next pass
  }
}

// Merge the split partials (Alg. 3 last two steps; see attn.hip for why this is a launch of its own).
__global__ __launch_bounds__(128) void attn_mla_combine_kernel(MlaParams p, int per_channel) {
  const int row = blockIdx.x;  // b*Hq + h
  const int b = row / p.Hq, h = row % p.Hq;
  const int64_t base = (int64_t)b * p.nsplit * p.Hq + h;
  float ms = -INFINITY;
  for (int s = 0; s < p.nsplit; ++s) ms = fmaxf(ms, p.part_m[base + (int64_t)s * p.Hq]);
  float l = 0.f;
  for (int s = 0; s < p.nsplit; ++s) {
    const float mv = p.part_m[base + (int64_t)s * p.Hq];
    if (mv != -INFINITY) l += p.part_l[base + (int64_t)s * p.Hq] * __builtin_amdgcn_exp2f(mv - ms);
  }
  for (int c = threadIdx.x; c < kLatV; c += 128) {
    float o = 0.f;
    for (int s = 0; s < p.nsplit; ++s) {
      const int64_t pr = base + (int64_t)s * p.Hq;
      const float mv = p.part_m[pr];
      if (mv != -INFINITY) o += p.part_o[pr * kLatV + c] * __builtin_amdgcn_exp2f(mv - ms);
    }
    float v = l > 0.f ? __fdiv_rn(o, l) : 0.f;
    if (per_channel) v *= p.scale[c];
    if (p.out_bf16)
      reinterpret_cast<uint16_t*>(p.out)[(int64_t)row * kLatV + c] = f32_to_bf16_bits(v);
    else
      reinterpret_cast<float*>(p.out)[(int64_t)row * kLatV + c] = v;
  }
}

int mla_nsplit(int B, int64_t L) { return attn_plan_nsplit(B, 1, L); }

}  // namespace

size_t attn_mla_workspace_bytes(int B, int Hq, int64_t L) {
  const size_t rows = (size_t)B * Hq * mla_nsplit(B, L);
  return align_up(rows * kLatV * 4, 256) + 2 * align_up(rows * 4, 256);
}

int launch_attn_mla(const AttnMlaArgs& a, hipStream_t stream) {
  MlaParams p{};
  p.q = a.q; p.C = a.C; p.scale = a.scale; p.kv_len = a.kv_len;
  p.B = a.B; p.Hq = a.Hq; p.L = a.L; p.ld = a.ld;
  p.nsplit = mla_nsplit(a.B, a.L);
  int64_t tps = cdiv(a.L > 0 ? a.L : 1, p.nsplit);
  tps = cdiv(tps, kAttnWaves * kTile) * (kAttnWaves * kTile);
  p.tokens_per_split = tps;
  p.sm_scale_log2 = a.sm_scale * kLog2e;
  const size_t rows = (size_t)a.B * a.Hq * p.nsplit;
  char* ws = (char*)a.workspace;
  p.part_o = (float*)ws;
  p.part_m = (float*)(ws + align_up(rows * kLatV * 4, 256));
  p.part_l = (float*)(ws + align_up(rows * kLatV * 4, 256) + align_up(rows * 4, 256));
  p.out = a.out;
  p.out_bf16 = a.out_bf16;
  if (a.taps) {
    p.tap_q1 = (int8_t*)a.taps->q1;
    p.tap_q2 = (int8_t*)a.taps->q2;
    p.tap_alpha = (float*)a.taps->scale;
    p.tap_s1 = a.taps->acc1;
    p.tap_s2 = a.taps->acc2;
    if (!(p.tap_q1 && p.tap_q2 && p.tap_alpha)) p.tap_q1 = p.tap_q2 = nullptr, p.tap_alpha = nullptr;
    if (!(p.tap_s1 && p.tap_s2)) p.tap_s1 = p.tap_s2 = nullptr;
  }
  constexpr size_t lds = (size_t)kAttnWaves * kLatHeads * kLatV * 4 + 2 * kLatHeads * kLatK +
                         kAttnWaves * 2 * kLatHeads * 64 + kLatHeads * 4 + 2 * kAttnWaves * kLatHeads * 4;
  const bool per_token = a.scale_mode == MSD_PER_TOKEN;
  static bool attr_set = false;
  if (!attr_set) {
    MSD_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_mla_kernel<true>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    MSD_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_mla_kernel<false>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_set = true;
  }
  const dim3 grid((unsigned)((int64_t)a.B * p.nsplit));
  if (per_token)
    hipLaunchKernelGGL((attn_mla_kernel<true>), grid, dim3(kAttnWaves * 64), lds, stream, p);
  else
    hipLaunchKernelGGL((attn_mla_kernel<false>), grid, dim3(kAttnWaves * 64), lds, stream, p);
  MSD_LAUNCH_CHECK();
  if (p.nsplit > 1) {
    hipLaunchKernelGGL(attn_mla_combine_kernel, dim3((unsigned)(a.B * a.Hq)), dim3(128), 0, stream, p,
                       per_token ? 0 : 1);
    MSD_LAUNCH_CHECK();
  }
  return MSD_OK;
}

}  // namespace msd
