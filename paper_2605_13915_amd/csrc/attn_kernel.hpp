// The MSD attention-decode kernel template and its launcher (see attn.hip for the method and the layout
// notes).  A header because the instantiations live in two translation units: attn.hip holds the ones for up
// to 8 query heads per KV head (two waves per SIMD), attn_wide.hip the ones that hold 16 or 24 heads per pass
// and is compiled with MFMA results placed in VGPRs (the merge code reads every result on the vector ALU;
// measured 4-9 % faster there and 2 % slower on the 8-head instances at long KV lengths).
#pragma once
#include "attn_common.hpp"

namespace msd {

// HPL = heads per lane group: 1 for G <= 4, 2 otherwise; an A fragment stacks 4*HPL heads x 2
// components (up to 16 rows).  NF = fragments held at once: 8*NF heads share one pass over the KV
// tiles -- the tiles, the V transposes and the scale of the P decomposition are per tile, everything
// from the score product to the running output is per fragment (NF = 2 and 3 need more than 256
// registers, i.e. one wave per SIMD).  MULTI: groups with more heads than that are processed 8*NF
// heads at a time, one walk over the workgroup's KV range each; without it the head loop has a
// single trip and disappears.
//
// LOWP: the low-precision arithmetic of Sec. 4.4 ("optimisation opportunities": decomposition and S / O
// merging in FP16 or integers instead of FP32) for the part of the kernel that runs on the vector ALU per
// (head, token):
//   S merge : alpha_Q S1 + beta_Q S2 = beta_Q (254 S1 + S2): one 24-bit integer multiply-add, one conversion,
//             one fp32 multiply (FP16 cannot hold S1, which reaches 127*127*128);
//   P codes : v = P~/alpha_P in [0, 127] is rounded once to FP16 and both passes run on packed FP16 pairs:
//             q1 = rne(v) as (v + 1536) - 1536 (the FP16 quantum at 1536 is 1), r = v - q1 (exact),
//             q2 = rne(254 r) as the fused 254 r + 1536 (the product is exact inside the FMA); the low byte of
//             the FP16 pattern of x + 1536 is the INT8 code of rne(x), so packing four codes is one byte
//             permute.  No clamp can fire (|254 r| <= 127).
//   O merge : alpha_P O1 + beta_P O2 = beta_P (254 O1 + O2), again one integer multiply-add and one conversion.
// Per element of P that is |v - (q1 + q2/254)| <= 2^-11 v + 1/508 in units of alpha_P instead of 1/508: the
// same for small probabilities, a relative 2^-11 for the largest ones.
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

template <int HPL, bool PER_TOKEN, bool MULTI, int NF, bool LOWP = false>
__global__ __launch_bounds__(kAttnWaves * 64) void attn_decode_kernel(AttnParams p, int nh_total) {
  constexpr int HF = 4 * HPL;  // heads per fragment
  constexpr int NH = HF * NF;  // head slots of one pass
  // LDS (dynamic): sO[waves][NH][kD] f32 | sP[waves][2][HF][16] u32 | sM[waves][NH] | sL[waves][NH] |
  // sAlpha[nh_total] | sQ[2][nh_total][kD] int8   (nh_total = G rounded up to a multiple of NH)
  extern __shared__ __attribute__((aligned(16))) uint8_t s_attn[];
  float(*sO)[NH][kD] = reinterpret_cast<float(*)[NH][kD]>(s_attn);
  uint32_t(*sP)[2][HF][16] = reinterpret_cast<uint32_t(*)[2][HF][16]>(s_attn + kAttnWaves * NH * kD * 4);
  float(*sM)[NH] = reinterpret_cast<float(*)[NH]>(s_attn + kAttnWaves * NH * kD * 4 + kAttnWaves * 2 * HF * 64);
  float(*sL)[NH] = sM + kAttnWaves;
  float* sAlpha = reinterpret_cast<float*>(sL + kAttnWaves);
  int8_t* sQ = reinterpret_cast<int8_t*>(sAlpha + nh_total);  // [comp][head][kD]: (comp * nh_total + head) * kD

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 15, g = lane >> 4;  // g: lane group = head group in D layouts; kg for operands
  const int bk = blockIdx.x / p.nsplit, split = blockIdx.x % p.nsplit;
  const int b = bk / p.Hkv, hk = bk % p.Hkv;
  const int G = p.G;
  int64_t len = p.kv_len ? (int64_t)p.kv_len[b] : p.L;
  len = max((int64_t)0, min(len, p.L));
  const int64_t t_begin = (int64_t)split * p.tokens_per_split;
  const int64_t t_end = min(len, t_begin + p.tokens_per_split);
  const int64_t kv_base = (int64_t)bk * p.L;  // token index base of this (b, kv head)
  const int8_t* Kb = p.K + kv_base * kD;
  const int8_t* Vb = p.V + kv_base * kD;

  // Tile loads are software-pipelined: the K/V/scale loads of the wave's next tile are issued
  // before the current tile is processed.  Token indices are clamped to the last valid token, so
  // every load is unconditional (a wave's look-ahead past its range re-reads that token).
  const int64_t last = max(t_end - 1, (int64_t)0);
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
  const int64_t t_first = t_begin + (int64_t)wave * kTile;
  // The first tile's loads go out before the query rows are decomposed: they do not depend on them, and a
  // split of a short cache is over after a few tiles, so the prologue's latency would otherwise show in full.
  // The loads of this wave's first query row are issued ahead of them (loads complete in order: the prologue
  // then waits for the query row only, not for the tile).
  uint32_t q_first = 0;
  float ks_first0 = 1.f, ks_first1 = 1.f;
  if (wave < G) {
    q_first = reinterpret_cast<const uint32_t*>(p.q + ((int64_t)b * p.Hq + hk * G + wave) * kD)[lane];
    if (!PER_TOKEN) {
      ks_first0 = p.k_scale[hk * kD + 2 * lane];
      ks_first1 = p.k_scale[hk * kD + 2 * lane + 1];
    }
  }
  if (t_first < t_end) load_tile(t_first, kfn, vrn, skn, svn);

  // ---- prologue: decompose the G query rows (Alg. 3 steps 1-2), one head per wave at a time
  for (int h = wave; h < nh_total; h += kAttnWaves) {
    uint32_t c1 = 0, c2 = 0;
    float alpha = 0.f;
    if (h < G) {
      const int64_t qrow = (int64_t)b * p.Hq + hk * G + h;
      const bool first = h == wave;  // loaded above
      const uint32_t w = first ? q_first : reinterpret_cast<const uint32_t*>(p.q + qrow * kD)[lane];
      float x0 = __uint_as_float(w << 16), x1 = __uint_as_float(w & 0xFFFF0000u);
      if (!PER_TOKEN) {  // absorb the per-channel K scale into Q
        x0 *= first ? ks_first0 : p.k_scale[hk * kD + 2 * lane];
        x1 *= first ? ks_first1 : p.k_scale[hk * kD + 2 * lane + 1];
      }
      const float mx = wave_max(fmaxf(fabsf(x0), fabsf(x1)));
      if (mx > 0.f) {
        alpha = __fdiv_rn(mx, 127.0f);
        const float beta = __fdiv_rn(alpha, 254.0f);
        int a0, b0, a1, b1;
        int8_codes(x0, alpha, beta, a0, b0);
        int8_codes(x1, alpha, beta, a1, b1);
        c1 = ((uint32_t)a0 & 0xFFu) | (((uint32_t)a1 & 0xFFu) << 8);
        c2 = ((uint32_t)b0 & 0xFFu) | (((uint32_t)b1 & 0xFFu) << 8);
      }
      if (split == 0 && p.tap_q1) {
        reinterpret_cast<uint16_t*>(p.tap_q1 + qrow * kD)[lane] = (uint16_t)c1;
        reinterpret_cast<uint16_t*>(p.tap_q2 + qrow * kD)[lane] = (uint16_t)c2;
        if (lane == 0) p.tap_alpha[qrow] = alpha;
      }
    }
    reinterpret_cast<uint16_t*>(sQ + (int64_t)h * kD)[lane] = (uint16_t)c1;
    reinterpret_cast<uint16_t*>(sQ + (int64_t)(nh_total + h) * kD)[lane] = (uint16_t)c2;
    if (lane == 0) sAlpha[h] = alpha;
  }
  __syncthreads();

  // A-fragment row of this lane (as an operand lane: row = j, k group = g)
  const int slot = j & 3;
  const bool row_valid = (HPL == 2) || (slot < 2);
  const int row_head = (j >> 2) * HPL + (HPL == 2 ? (slot >> 1) : 0);  // head within the fragment
  const int row_comp = (HPL == 2) ? (slot & 1) : slot;
  const v4i zero4 = {0, 0, 0, 0};
  const float sm_scale = kLog2e / sqrtf((float)kD);  // scores are kept in log2 units

  for (int h0 = 0; h0 < (MULTI ? G : 1); h0 += NH) {  // one pass over the KV range per NH heads
  v4i qa[NF][2];
#pragma unroll
  for (int f = 0; f < NF; ++f)
#pragma unroll
    for (int s = 0; s < 2; ++s)
      qa[f][s] = (row_valid && h0 + f * HF + row_head < G)
                     ? *reinterpret_cast<const v4i*>(sQ + (int64_t)(row_comp * nh_total + h0 + f * HF + row_head) * kD +
                                                     64 * s + 16 * g)
                     : zero4;
  // per-lane-group state (as a D lane: head h0 + f*HF + g*HPL + hh)
  float aq[NF][HPL], bq[NF][HPL], m_run[NF][HPL], l_run[NF][HPL], o_run[NF][HPL][8];
#pragma unroll
  for (int f = 0; f < NF; ++f)
#pragma unroll
    for (int hh = 0; hh < HPL; ++hh) {
      aq[f][hh] = sAlpha[h0 + f * HF + g * HPL + hh];
      bq[f][hh] = __fdiv_rn(aq[f][hh], 254.0f);
      m_run[f][hh] = -INFINITY;
      l_run[f][hh] = 0.f;
#pragma unroll
      for (int c = 0; c < 8; ++c) o_run[f][hh][c] = 0.f;
    }
  if (h0 > 0 && t_first < t_end) load_tile(t_first, kfn, vrn, skn, svn);  // (the first pass: before the prologue)
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
    // scale of the P decomposition: alpha_P = top/127 with top a bound on P (or P*s_V)
    float top = 1.f;
    if (PER_TOKEN) top = row16_max(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])));
    const bool coded = top > 1e-30f;  // below that every code of the tile is zero (and 127 / top would overflow)
    const float to_code = coded ? __fdiv_rn(127.0f, top) : 0.f;
    const float from_code = coded ? top * (1.0f / 127.0f) : 0.f;
    uint32_t vb[8][4];  // filled by the first fragment of the tile
#pragma unroll
    for (int f = 0; f < NF; ++f) {
      // ---- (2) S1, S2 for the heads of this fragment
      v4i sd[4];
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) {
        sd[tt] = mfma_s8(qa[f][0], kf[tt][0], zero4);
        sd[tt] = mfma_s8(qa[f][1], kf[tt][1], sd[tt]);
      }
      if (p.tap_s1) {
#pragma unroll
        for (int hh = 0; hh < HPL; ++hh) {
          const int head = h0 + f * HF + g * HPL + hh;
          if (head < G) {
            const int64_t row = ((int64_t)b * p.Hq + hk * G + head) * p.L;
#pragma unroll
            for (int tt = 0; tt < 4; ++tt)
              if (live[tt]) {
                p.tap_s1[row + t0 + 16 * tt + j] = sd[tt][2 * hh];
                p.tap_s2[row + t0 + 16 * tt + j] = sd[tt][2 * hh + 1];
              }
          }
        }
      }
      // ---- (3)+(4) merge, online softmax, decompose P
      float corr[HPL];
      uint32_t pk1[HPL], pk2[HPL];
#pragma unroll
      for (int hh = 0; hh < HPL; ++hh) {
        float s[4];
        float mx = -INFINITY;
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
          float v;
          if (LOWP)  // |S1| < 2^21: the 24-bit multiply is exact
            v = (float)(__mul24(sd[tt][2 * hh], 254) + sd[tt][2 * hh + 1]) * (bq[f][hh] * (sm_scale * sk[tt]));
          else
            v = (aq[f][hh] * (float)sd[tt][2 * hh] + bq[f][hh] * (float)sd[tt][2 * hh + 1]) * (sm_scale * sk[tt]);
          s[tt] = live[tt] ? v : -INFINITY;
          mx = fmaxf(mx, s[tt]);
        }
        mx = row16_max(mx);
        const float m_new = fmaxf(m_run[f][hh], mx);
        corr[hh] = __builtin_amdgcn_exp2f(m_run[f][hh] - m_new);
        m_run[f][hh] = m_new;
        float lsum = 0.f;
        uint32_t w1 = 0, w2 = 0;
        if (LOWP) {
          float t[4];
#pragma unroll
          for (int tt = 0; tt < 4; ++tt) {
            const float pr = __builtin_amdgcn_exp2f(s[tt] - m_new);
            lsum += pr;
            t[tt] = pr * sv[tt] * to_code;  // P (times s_V) in units of alpha_P, in [0, 127]
          }
          const half2_t magic = {(_Float16)1536.0f, (_Float16)1536.0f}, k254 = {(_Float16)254.0f, (_Float16)254.0f};
          uint32_t m1[2], m2[2];
#pragma unroll
          for (int pr2 = 0; pr2 < 2; ++pr2) {
            const half2_t vh = {(_Float16)t[2 * pr2], (_Float16)t[2 * pr2 + 1]};  // the one rounding to FP16
            const half2_t a1 = vh + magic;      // integer part in the low mantissa bits
            const half2_t c1 = a1 - magic;      // rne(vh), exact
            const half2_t a2 = __builtin_elementwise_fma(vh - c1, k254, magic);  // one rounding: rne(254 r) exactly
            m1[pr2] = __builtin_bit_cast(uint32_t, a1);
            m2[pr2] = __builtin_bit_cast(uint32_t, a2);
          }
          // byte 0 of each half: codes of tokens tt = 0..3 in bytes 0..3
          w1 = __builtin_amdgcn_perm(m1[1], m1[0], 0x06040200u);
          w2 = __builtin_amdgcn_perm(m2[1], m2[0], 0x06040200u);
        } else {
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
          const float pr = __builtin_amdgcn_exp2f(s[tt] - m_new);
          lsum += pr;
          const float t = pr * sv[tt] * to_code;  // P (times s_V) in units of alpha_P
          const float c1 = fminf(rintf(t), 127.f);
          const float c2 = fminf(fmaxf(rintf((t - c1) * 254.0f), -127.f), 127.f);
          w1 |= ((uint32_t)(int)c1 & 0xFFu) << (8 * tt);
          w2 |= ((uint32_t)(int)c2 & 0xFFu) << (8 * tt);
        }
        }
        l_run[f][hh] = l_run[f][hh] * corr[hh] + lsum;
        pk1[hh] = w1;
        pk2[hh] = w2;
        if (p.tap_p1) {  // observation points only
          const int head = h0 + f * HF + g * HPL + hh;
          if (head < G) {
            const int64_t row = ((int64_t)b * p.Hq + hk * G + head) * p.L;
#pragma unroll
            for (int tt = 0; tt < 4; ++tt)
              if (live[tt]) {
                p.tap_p1[row + t0 + 16 * tt + j] = (int8_t)(w1 >> (8 * tt));
                p.tap_p2[row + t0 + 16 * tt + j] = (int8_t)(w2 >> (8 * tt));
              }
          }
        }
      }
      // ---- hand P to the A-fragment layout through LDS (wave-private)
#pragma unroll
      for (int hh = 0; hh < HPL; ++hh) {
        sP[wave][0][g * HPL + hh][j] = pk1[hh];
        sP[wave][1][g * HPL + hh][j] = pk2[hh];
      }
      __builtin_amdgcn_wave_barrier();
      const v4i pa = row_valid ? *reinterpret_cast<const v4i*>(&sP[wave][row_comp][row_head][4 * g]) : zero4;
      __builtin_amdgcn_wave_barrier();
      // ---- V_t into token-contiguous B fragments: vb[c][jq] = 4 token bytes of channel 8j+c
      if (f == 0) {
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
      }
      // ---- (5) O1, O2, merge and rescale the running output
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const v4i bf = {(int)vb[c][0], (int)vb[c][1], (int)vb[c][2], (int)vb[c][3]};
        const v4i od = mfma_s8(pa, bf, zero4);
#pragma unroll
        for (int hh = 0; hh < HPL; ++hh) {
          const float ot = LOWP ? (from_code * (1.0f / 254.0f)) * (float)(__mul24(od[2 * hh], 254) + od[2 * hh + 1])
                                : from_code * ((float)od[2 * hh] + (float)od[2 * hh + 1] * (1.0f / 254.0f));
          o_run[f][hh][c] = o_run[f][hh][c] * corr[hh] + ot;
        }
      }
      // keep the fragments apart in the schedule: interleaving them multiplies the live registers
      if (NF > 1) __builtin_amdgcn_sched_barrier(0);
    }
  }

  // ---- merge the waves of this workgroup, write the split's partial (m, l, O) of these heads
#pragma unroll
  for (int f = 0; f < NF; ++f)
#pragma unroll
    for (int hh = 0; hh < HPL; ++hh) {
      const float lt = row16_sum(l_run[f][hh]);
      const int hs = f * HF + g * HPL + hh;
      if (j == 0) {
        sM[wave][hs] = m_run[f][hh];
        sL[wave][hs] = lt;
      }
#pragma unroll
      for (int c = 0; c < 8; ++c) sO[wave][hs][8 * j + c] = o_run[f][hh][c];
    }
  __syncthreads();
  const int nh_here = min(NH, G - h0);
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
    if (p.nsplit == 1) {  // no cross-workgroup step at all
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
  if (MULTI && h0 + NH < G) __syncthreads();  // the merge buffers are reused by the next head group
  }
}

template <int HPL, bool PER_TOKEN, bool MULTI, int NF, bool LOWP = false>
int launch_attn_variant(const AttnParams& p, dim3 grid, hipStream_t stream) {
  constexpr int HF = 4 * HPL, NH = HF * NF;
  const int nh_total = (int)cdiv(p.G, NH) * NH;
  const size_t lds = (size_t)kAttnWaves * NH * kD * 4 + kAttnWaves * 2 * HF * 64 + 2 * kAttnWaves * NH * 4 +
                     (size_t)nh_total * 4 + (size_t)2 * nh_total * kD;
  static size_t attr_bytes = 64 * 1024;
  if (lds > attr_bytes) {
    MSD_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_decode_kernel<HPL, PER_TOKEN, MULTI, NF, LOWP>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_bytes = lds;
  }
  hipLaunchKernelGGL((attn_decode_kernel<HPL, PER_TOKEN, MULTI, NF, LOWP>), grid, dim3(kAttnWaves * 64), lds, stream, p, nh_total);
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

}  // namespace msd
